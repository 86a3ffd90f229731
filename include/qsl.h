/* qsl.h -- C ABI of the MI355X-native compression hot path of Qsparse-local-SGD
 * (Basu, Data, Karakus, Diggavi, arXiv:1906.02367).
 *
 * The library computes, for R simulated workers held as a batch on ONE GPU, the two worker
 * lines and the master line of a synchronisation step of Algorithm 1:
 *
 *     g^(r)  <-  Q Comp_k( m^(r) + Delta^(r) )          (compress, "send")
 *     m^(r)  <-  m^(r) + Delta^(r) - g^(r)              (error memory update)
 *     x      <-  x - (1/R) sum_r g^(r)                   (aggregate at the master)
 *
 * with Comp_k in {Top_k, Rand_k} (Section 2.2), Q in {QSGD with s levels (Definition 1,
 * example 1), Sign scaled by ||Comp_k(x)||_1 / k (Definition 2, Lemma 3 with m = 1)}, the
 * quantiser acting on the k kept values as a length-k vector (proof of Lemma 1), and the whole
 * operator optionally applied block by block (Corollary 1).
 *
 * Conventions
 *   - Every `device` pointer is GPU memory owned by the caller; [R, d] arrays are row-major,
 *     contiguous, row stride d; message arrays are [R, qsl_msg_capacity_bytes()] bytes.
 *     Device pointers must be 4-byte aligned (messages and 64-bit outputs 8-byte aligned).
 *   - `host` pointers are ordinary CPU memory, read (or written) before the call returns.
 *   - All GPU work is enqueued on the context's HIP stream and is asynchronous; nothing on the
 *     hot path allocates, frees or synchronises.  The context owns only scratch memory.
 *   - Argument errors are reported synchronously and have no side effect.  Errors that depend
 *     on the data (a NaN/Inf in m + Delta) set a status word on the device, returned by
 *     qsl_device_status().
 *   - A context is not thread-safe; calls on one context must not overlap on the host.  On the GPU the
 *     calls of one context share its scratch memory and are ordered by its stream; when the stream is
 *     changed (qsl_set_stream) the library makes the new stream wait for the work already enqueued on
 *     the old one, so calls on different streams still run one after the other.
 *
 * Wire format of one message (little endian; fields are packed least-significant bit first;
 * "w_idx" = bits needed to write d - 1, at least 1; "w_lev" = bits needed to write s - 1):
 *     u32  nnz                         number of transmitted coordinates
 *     f32  scale[num_segments]         per segment: ||v_S||_2 (QSGD), ||v_S||_2 / (1 + beta) (scaled QSGD),
 *                                      ||v_S||_1 / k or ||v_S||_2 / k (Sign), 0 (no quantiser)
 *     u32  nnz_l[num_segments]         only for QSGD (either form) with num_segments > 1
 *     nnz x w_idx bits                 coordinate indices, ascending     (starts on a 32-bit boundary)
 *     nnz x w_val bits                 QSGD: (level - 1) in w_lev bits, then the sign bit;
 *                                      Sign: the sign bit (1 = negative); no quantiser: the fp32 value
 *                                      (starts on a 32-bit boundary)
 *     zero padding up to the capacity (a multiple of 8 bytes)
 * Index-free format (QSL_FLAG_DENSE_FORMAT; every coordinate is kept, so entry j is coordinate j):
 *     u32  d
 *     f32  scale[num_segments]
 *     d x w_code bits                  QSGD: the level 0..s in the bits needed to write s, then the sign bit;
 *                                      Sign: the sign bit; no quantiser: the fp32 value
 *     zero padding up to the capacity
 *   payload bits = 32 + 32 num_segments + d w_code.
 * A QSGD coordinate whose level is 0 is not transmitted (Section 5.1.2 observes that the
 * quantiser adds sparsity of its own).  The paper fixes no encoding; this one is the library's choice.
 */
#ifndef QSL_H
#define QSL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct qsl_ctx qsl_ctx;

typedef enum {
  QSL_OK = 0,
  QSL_ERR_INVALID_ARG = 1,
  QSL_ERR_BUFFER_TOO_SMALL = 2,
  QSL_ERR_NONFINITE_INPUT = 3,
  QSL_ERR_DEVICE = 4,
  QSL_ERR_UNSUPPORTED = 5
} qsl_status;

enum { QSL_TOPK = 0, QSL_RANDK = 1 };    /* sparsifier, Section 2.2 */
/* quantiser: QSGD (Definition 1, example 1); Sign scaled by ||Comp_k(x)||_1 / k (Definition 2, Lemma 3
 * with m = 1), by ||Comp_k(x)||_2 / k (m = 2), or by ||Comp_k(x)||_m / k with m = 3, 4 (QSL_SIGN_L3, QSL_SIGN_L4: the
 * exact sum of the m-th powers rounded to double, its root in double -- two square roots for m = 4, for m = 3 a start
 * value from the binary exponent and eight Newton steps, every step one IEEE operation -- divided by k in double and
 * rounded to float); none, i.e. Comp_k(x) itself in fp32 (the
 * TopK-SGD comparison scheme of Section 5); QSGD divided by 1 + beta_{k,s}, beta_{k,s} = min(k/s^2,
 * sqrt(k)/s) (the scaled composition of Lemma 2: same level codes, transmitted norm N / (1 + beta)). */
enum { QSL_QSGD = 0, QSL_SIGN_L1 = 1, QSL_SIGN_L2 = 2, QSL_FP32 = 3, QSL_QSGD_SCALED = 4, QSL_SIGN_L3 = 5, QSL_SIGN_L4 = 6 };

/* Parameters of the operator Q Comp_k, in the paper's notation. */
typedef struct {
  uint64_t d;                 /* coordinates per worker, 1 <= d < 2^32                                  */
  uint32_t num_segments;      /* 1: one operator on the whole vector; 1 < L <= 16384: piecewise (Cor. 1)  */
  const uint64_t *seg_offset; /* host, num_segments + 1 entries, seg_offset[0] = 0, last = d, increasing */
  const uint32_t *seg_k;      /* host, k per segment, 1 <= k_l <= size of the segment                   */
  uint32_t s;                 /* QSGD levels, 1 <= s <= 32768 (ignored by the other quantisers)         */
  uint32_t sparsifier;        /* QSL_TOPK or QSL_RANDK                                                  */
  uint32_t quantizer;         /* one of the QSL_QSGD .. QSL_QSGD_SCALED values above                    */
  uint64_t seed;              /* seed of the counter-based randomness (Rand_k choice, QSGD rounding)    */
  uint32_t max_workers;       /* largest R passed to one call; scratch is sized for it                  */
  uint32_t flags;             /* 0, or QSL_FLAG_* below                                                 */
} qsl_config;

enum {
  QSL_FLAG_NO_FAST_PATH = 1,  /* never guess a threshold and never skip the selection of a segment with k = size:
                                 exact multi-pass selection only (testing, comparison)                  */
  QSL_FLAG_NO_SMALL_PATH = 2, /* segments of at most 4096 coordinates also take the multi-pass kernels
                                 instead of the one-block selection (testing, comparison)               */
  QSL_FLAG_NO_WARM_START = 8, /* every call guesses its thresholds from a fresh sample of m + delta, as the first call
                                 does, instead of taking them from the previous call's candidates (testing, comparison) */
  QSL_FLAG_DENSE_FORMAT = 16, /* only for an operator that keeps every coordinate (k = size in every segment: the
                                 error-feedback schemes without sparsification that Section 5 compares with): the
                                 messages have the index-free format described above, and qsl_compress runs as two
                                 streaming passes                                                        */
  QSL_FLAG_OWN_V = 4          /* the context also allocates a float [max_workers, d] array of its own as the home
                                 of v = m + delta, so that qsl_compress / qsl_compress_diff accept m_out = NULL
                                 ("send g, leave the error memory alone")                               */
};

/* Which way each segment of an operator will take through the selection -- the `path` that qsl_debug_units
 * reports, before any failed guess: 0 = single-pass with a guessed threshold, 1 = multi-pass, 3 = one block,
 * 4 = no selection (k = size).  The decision depends on (size, k, sparsifier, flags) only; qsl_create makes it
 * with the same code.  Needs no context and no GPU.
 *   cfg host; path_out host, uint32 [num_segments] */
qsl_status qsl_plan_paths(const qsl_config *cfg, uint32_t *path_out);

/* Create a context for one operator on the current HIP device.  `hip_stream` is a hipStream_t
 * (NULL = the default stream).  Allocates all scratch memory.  */
qsl_status qsl_create(qsl_ctx **out, const qsl_config *cfg, void *hip_stream);
qsl_status qsl_destroy(qsl_ctx *ctx);
/* Later calls are enqueued on `hip_stream`.  If it differs from the current stream, the new stream first waits
 * (hipStreamWaitEvent, no host synchronisation) for everything this context has enqueued on the old one.  */
qsl_status qsl_set_stream(qsl_ctx *ctx, void *hip_stream);

/* Size in bytes of one worker's message buffer (an upper bound over all inputs; multiple of 8). */
size_t qsl_msg_capacity_bytes(const qsl_ctx *ctx);

/* Algorithm 1, worker lines of a synchronisation step, for workers worker0 .. worker0 + R - 1 at
 * sync round `round` (< 2^62): forms v = m + delta, selects, quantises, packs the messages and
 * writes the new error memory.
 *   m, delta  device, const float [R, d]
 *   m_out     device, float [R, d]; receives m + delta - g; may be the same pointer as m.  NULL only for a
 *             context created with QSL_FLAG_OWN_V: the messages are produced and m is left as it was
 *             (the error update can follow later with qsl_error_update)
 *   msg       device, uint8 [R, capacity]; every byte is written (zero padded)
 *   msg_bits  device, uint64 [R] or NULL; payload bits of each message (padding excluded)
 *   sel_idx   device, uint32 [R, K] or NULL, K = sum_l k_l; the selected coordinates, ascending
 *   sel_level device, uint16 [R, K] or NULL; QSGD level 0..s of each selected coordinate
 *             (0 = not transmitted); 1 for every entry under the sign quantiser
 * The random word of coordinate i is Philox4x32-10 with counter (i / 4, worker, round mod 2^32,
 * (round >> 32) | stream << 30), key (seed mod 2^32, seed >> 32), output word i mod 4; stream 0
 * ranks coordinates for Rand_k, stream 1 drives the QSGD rounding.
 * Speed only, never the result: for Top_k the context keeps, per row r of the batch and per segment, a guess of
 * the selection threshold taken from its previous call (the first call, or QSL_FLAG_NO_WARM_START, samples the
 * input instead).  The guess serves best when row r carries the same worker from call to call; a context
 * whose rows change hands between unrelated inputs selects just as exactly, but may do so by slower kernels.  */
qsl_status qsl_compress(qsl_ctx *ctx, const float *m, const float *delta, float *m_out, uint32_t worker0,
                        uint32_t R, uint64_t round, uint8_t *msg, uint64_t *msg_bits, uint32_t *sel_idx,
                        uint16_t *sel_level);

/* The same step with the difference of Algorithm 1's synchronisation line formed on the fly:
 * Delta = x_t - xhat_{t+1/2} is computed in registers (one fp32 subtraction per coordinate, then
 * v = m + Delta as above), so the caller never materialises Delta.  Bit for bit the result of
 * qsl_compress on delta[r, j] = x[j] - xhat_half[r, j].
 *   x          device, const float [d]; the master's model, shared by the R workers
 *   xhat_half  device, const float [R, d]; the local models after the local step
 * Neither may overlap m_out.  All other arguments as for qsl_compress.  */
qsl_status qsl_compress_diff(qsl_ctx *ctx, const float *m, const float *x, const float *xhat_half, float *m_out,
                             uint32_t worker0, uint32_t R, uint64_t round, uint8_t *msg, uint64_t *msg_bits,
                             uint32_t *sel_idx, uint16_t *sel_level);

/* Algorithm 1, second worker line on its own: m <- (m + delta) - decode(msg), in place, for R
 * workers.  Gives bit-for-bit the memory that qsl_compress writes to m_out.
 *   m device float [R, d] (updated), delta device const float [R, d], msg device const [R, capacity] */
qsl_status qsl_error_update(qsl_ctx *ctx, float *m, const float *delta, const uint8_t *msg, uint32_t R);

/* Algorithm 1, master line (and Algorithm 2's, where only a subset reports and the scale stays
 * 1/R):  out[j] = (accumulate ? out[j] : 0) + scale * sum_{r in list, in list order} decode(msg_r)[j],
 * the inner sum accumulated in fp32 in list order, without atomics.
 *   msg          device const uint8 [*, capacity]
 *   worker_list  host, R row numbers into msg, or NULL for rows 0 .. R-1;  R <= 64
 *   out          device float [d]                                                     */
qsl_status qsl_aggregate(qsl_ctx *ctx, const uint8_t *msg, const uint32_t *worker_list, uint32_t R, float scale,
                         int accumulate, float *out);

/* For callers that cannot allocate (code under HIP graph capture, serving loops, harnesses that forbid
 * hipMalloc): the master line as qsl_aggregate computes it, without a context and without any allocation.
 * The scratch of the aggregation kernels (one directory per listed message, and the status word) lives in a
 * fixed array of device memory inside the library, QSL_STATIC_SCRATCH_BYTES per GPU, held until the process
 * ends.  Same kernels, same order of additions and same result, bit for bit, as qsl_aggregate on a context
 * created from `cfg`.
 *   cfg          host; one segment only (num_segments = 1: a piecewise operator needs its segment tables in
 *                device memory); seed, max_workers and flags are ignored
 *   hip_stream   the stream to enqueue on (NULL = the default stream)
 *   msg, worker_list, R, scale, accumulate, out   as for qsl_aggregate
 * QSL_ERR_UNSUPPORTED if num_segments > 1 or if rows * (ceil(d / 1024) + 1) * 4 + 256 bytes exceed the array, where
 * rows = 65 when the kernels for many messages are used (R >= 56, or R >= 24 with long messages), else R;
 * QSL_ERR_DEVICE if the device's ordinal is 64 or more.  Entries with an index >= d are skipped silently.
 * All calls on one GPU share the array: calls that overlap on one GPU (two streams, two threads) race.  */
#define QSL_STATIC_SCRATCH_BYTES (8u << 20)
qsl_status qsl_aggregate_static(const qsl_config *cfg, void *hip_stream, const uint8_t *msg,
                                const uint32_t *worker_list, uint32_t R, float scale, int accumulate, float *out);

/* Payload bits of each of R messages (the communication-budget axis of the plots of Section 5: test
 * error and loss against the number of bits sent), read from the message headers.  Synchronises the stream.  bits_host: host uint64 [R].  */
qsl_status qsl_bits_sent(qsl_ctx *ctx, const uint8_t *msg, uint32_t R, uint64_t *bits_host);

/* Accounting variant for Rand_k: the bits of one message if the indices are not transmitted.  Rand_k
 * (Section 2.2) chooses its k-subset independently of the data, so a receiver that shares the seed and
 * knows the worker and the round can regenerate it; the message then carries, per segment, the fp32
 * scale, and per selected coordinate one fixed-width code: QSGD the level 0..s and a sign bit (level 0
 * must now be written, the position is no longer free to drop), Sign one bit, no quantiser 32 bits.
 * Needs no context and no GPU.  QSL_ERR_UNSUPPORTED for Top_k (its support depends on the data).
 * The library does not emit this format; the count is for the communication axis of the paper's plots.
 *   cfg host; bits host, receives the count */
qsl_status qsl_bits_index_free(const qsl_config *cfg, uint64_t *bits);

/* Synchronise the stream and return QSL_ERR_NONFINITE_INPUT if any compress call since the last
 * query met a NaN or Inf in m + delta (its outputs are then unspecified), QSL_ERR_DEVICE on a HIP
 * error or if a kernel met a malformed message (an index >= d; the entry is skipped), else QSL_OK.
 * Clears the word.  */
qsl_status qsl_device_status(qsl_ctx *ctx);

/* Per-unit diagnostics of the last compress call (unit = worker-major (worker, segment)); synchronises.
 * out_host receives, per unit, 8 uint32: {path, candidates, threshold key, n_greater, n_equal_taken,
 * guess key, scale bits, transmitted}; path: 0 = single-pass fast path, 1 = multi-pass path by
 * configuration, 2 = multi-pass path after a failed guess, 3 = one-block selection of a small segment,
 * 4 = no selection (k equals the size of the segment: every coordinate is kept).  */
qsl_status qsl_debug_units(qsl_ctx *ctx, uint32_t *out_host, uint32_t max_units, uint32_t *n_units);

/* Kernel timing for the benchmark: when enabled, compress calls bracket the streaming kernel with
 * HIP events on the context's stream.  qsl_timing_read synchronises, returns the summed duration
 * in milliseconds and the number of bracketed launches since it was enabled, and resets both.  */
qsl_status qsl_timing_enable(qsl_ctx *ctx, int enabled);
qsl_status qsl_timing_read(qsl_ctx *ctx, double *total_ms, uint32_t *launches);

const char *qsl_status_string(qsl_status st);

#ifdef __cplusplus
}
#endif
#endif /* QSL_H */
