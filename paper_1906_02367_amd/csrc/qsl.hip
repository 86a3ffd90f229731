// qsl.hip -- kernels and C ABI of the compression hot path of Qsparse-local-SGD for gfx950.
//
// One synchronisation step of Algorithm 1 (arXiv:1906.02367) for a batch of R workers:
//   k_sample     the guess (Top_k only): a quantile of a strided sample of |m + Delta| (of group maxima
//                of the whole unit when no sample is reliable); for Rand_k the rank keys are uniform
//                random words, so the guess is analytic
//   k_stream     v = m + Delta (worker line 1), written over the error memory in ONE pass over HBM;
//                each wave streams one chunk of 1024 coordinates and leaves the coordinates whose
//                rank key reaches the unit's guess in the chunk's own slot line (written as one
//                full 128-byte line: no read-modify-write in HBM, no atomic to wait for)
//   k_select<l>  exact radix selection of the k-th largest key (Section 2.2: Top_k / Rand_k), 12+12+8
//                bits, over the candidates -- or over the whole vector when the guess failed or the
//                unit is too dense for guessing (the general path; always exact)
//   k_small      a unit of at most 4 chunks: selection, ordered compaction and norm by one block
//   k_tile_count / k_tile_write    ordered compaction of the selected coordinates, ties to the lower index
//                (k_tile_write also accumulates the exact ||v_S||_2^2 or ||v_S||_1: proof of Lemma 1; Lemma 3, m = 1)
//   k_quantize   QSGD levels (Definition 1, example 1) or signs (Definition 2); error update
//                m <- v - g on the transmitted coordinates (Algorithm 1, worker line 2)
//   k_surv_compact, k_pack    the packed message
//   k_aggregate  master line of Algorithm 1, atomic-free
//
// A "unit" is one (worker, segment) pair: the operator is applied independently to each unit
// (Corollary 1).  Rank key: Top_k: magnitude bits of v shifted left by one; Rand_k: the
// coordinate's random word of stream 0.  Larger key first, ties to the lower coordinate.
//
// No kernel waits for another block and none uses a device-wide fence (on this GPU the L2 is per
// XCD, so a device-scope release costs a cache write-back): a value that needs all blocks of a
// unit -- the radix digit, a prefix of block counts, the fp32 scale -- is recomputed by every block
// of the NEXT kernel from the small per-block results the previous one left in memory.  Counters
// that many waves add to sit in cache lines of their own: atomics that share a line serialise.
//
// Arithmetic contract: every fp32 operation that decides an output is a single IEEE operation
// (compile with -ffp-contract=off, no fast-math); norms are the exact sum rounded once to double.

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "qsl.h"
#include "qsl_device.h"

using namespace qsl;

namespace {

constexpr uint32_t CHUNK = 1024;           // coordinates one wave streams: 4 x (64 lanes x 4)
constexpr uint32_t BLOCK = 256;
constexpr uint32_t HBINS = 4096;           // radix digits: 12 + 12 + 8 bits of the 32-bit rank key
constexpr uint32_t ACC_SLOTS = 20;         // 32-bit digits of the exact accumulator
constexpr uint32_t MAX_SAMPLE_BLOCKS = 128; // blocks (of 1024 threads) per unit of the sampling kernel: 1 .. 128
constexpr uint32_t MAX_SELECT_BLOCKS = 64; // blocks (of 1024 threads) per unit of the selection kernels: 1 .. 64
constexpr uint32_t BIG = 1024;             // threads of the sampling and selection kernels
constexpr uint32_t MAX_QB_INLINE = 4096;   // above this many quantise blocks a separate prefix kernel runs
constexpr uint32_t NSUB = 64;              // candidate counters per unit: chunk t adds to counter t mod 64
constexpr uint32_t PAD = 64;               // words between two counters: atomics that share a cache line serialise
constexpr uint32_t CTR_OVF = NSUB;         // counter NSUB: cursor of the unit's overflow pool
constexpr uint32_t CTR_FAIL = NSUB + 1;    // counter NSUB + 1: set when the overflow pool ran out
constexpr uint32_t CTR_LINES = NSUB + 2;

enum : uint32_t { PATH_FAST = 0, PATH_GENERAL = 1, PATH_FALLBACK = 2, PATH_SMALL = 3 };
constexpr uint32_t SMALL_CHUNKS = 4;       // a unit of at most 4 chunks (4096 coordinates) is selected by one block

struct SegInfo {
  uint64_t start, size;
  uint64_t slot_off;     // first slot element (uint2) of this segment inside one worker's slot area
  uint64_t ovf_off;      // first entry of this segment inside one worker's overflow pool
  uint64_t d0_off;       // first entry of this segment inside one worker's dense candidate lists
  uint32_t k, koff;      // koff: first slot in the [K] selected arrays
  uint32_t nwt;          // chunks of 1024 coordinates
  uint32_t d0_cap;       // entries of the dense candidate list
  uint32_t wc_base;      // first per-wave counter of this segment (per worker)
  uint32_t cb_base, ncb; // compaction blocks: index of the first one (per worker), how many
  uint32_t nsamp;        // blocks of this unit in the sampling kernel
  uint32_t mode;         // PATH_FAST, PATH_GENERAL or PATH_SMALL, decided on the host from (size, k)
  uint32_t lpc;          // slot size: lpc * 16 bytes per chunk (4: 64 bytes, 8: one 128-byte line, 16: two lines)
  uint32_t ovf_cap;      // entries of the overflow pool
  uint32_t n_runs;       // sample: runs of 64 consecutive coordinates
  uint32_t r_s;          // sample rank that defines the guess
  uint32_t T_static;     // Rand_k: analytic guess
  uint32_t nsel;         // blocks of this unit in the selection kernels
  uint32_t samp_stride;  // sample: distance between the starts of two runs (64: the whole unit is read)
};

struct WtInfo { uint32_t seg, chunk, pad0, pad1; };                 // one chunk (multi-segment contexts only)
struct SelInfo { uint32_t seg, j, pad0, pad1; };                    // one block of a selection kernel
struct CbInfo { uint32_t seg, b, pad0, pad1; };                     // one compaction block

// Every field is written by exactly one kernel of a call and read only by later kernels (the blocks of
// one launch start at different times: a field that a launch both reads and rewrites would show late
// blocks the new value).
struct UnitState {
  uint32_t path;        // static: PATH_FAST, PATH_GENERAL or PATH_SMALL
  uint32_t T;           // guess key (k_sample_scan; static for Rand_k and for the general path)
  uint32_t cand;        // candidates collected (k_select<0>)
  uint32_t fell_back;   // 1: the guess failed, the unit runs the general path (k_select<0>)
  uint32_t prefix1, k_rem1; // radix selection state after the first digit (found by k_select<1> from the first histogram) ...
  uint32_t prefix2, k_rem2; // ... and after the second (k_select<2>); the third is found by k_tile_count
  uint32_t tau, need, n_gt; // threshold key, how many equal to it are kept, how many above (k_tile_count)
  uint32_t nnz;         // transmitted coordinates (zeroed by k_select<0>, counted by k_quantize)
  uint32_t scale_bits;  // fp32 scale (k_quantize)
  uint32_t pad;
};

struct DevCtx {
  const SegInfo* segs; const WtInfo* wts; const SelInfo* sels; const SelInfo* samps; const CbInfo* cbs;
  const uint32_t* fast_segs;
  const uint32_t* small_segs;
  const uint32_t* big_segs; // the segments that are not selected by one block (they use histograms)
  const uint32_t* seg_dir;  // [ceil(d / 1024) + 1]: segment of coordinate t * 1024 (the last entry: L - 1)
  const uint32_t* slot_dir; // [ceil(K / 256) + 1]: segment of slot b * 256 of the selected arrays
  UnitState* units;
  uint2* slots; uint64_t slot_stride;   // per worker: one slot (lpc * 2 elements) per chunk of every fast segment
  uint2* ovf; uint64_t ovf_stride;      // per worker: overflow pools, for chunks with more candidates than a slot holds
  uint32_t* slot_key; uint32_t* ovf_key; // Rand_k only: the rank key (random word) of every slot element / pool entry
  uint2* d0; uint32_t* d0_key; uint64_t d0_stride;   // per worker: dense, coordinate-ordered candidate lists (+ keys, Rand_k)
  uint32_t* wave_cnt;   // [R][NWC]: candidates met by each wave of k_select<0>
  uint2* cb_cnt;        // [R][NCB]: (#key > tau, #key == tau) of each compaction block
  uint32_t* hist;       // [U][3][HBINS], one histogram per radix digit; all zero between calls
  uint32_t* ctr;        // [U][CTR_LINES][PAD]; word 0 of each line is a counter; all zero between calls
  uint64_t* norm_acc;   // [U][ACC_SLOTS]; all zero between calls
  uint32_t* sel_idx; uint32_t* sel_val; uint32_t* sel_code;   // [R][K]; code = level | neg << 31
  uint32_t* blk_cnt;    // [R][QB] survivors per quantise block
  uint32_t* blk_pre;    // [R][QB + 1] their exclusive prefix and total (only when QB > MAX_QB_INLINE)
  uint32_t* surv_idx; uint32_t* surv_code;                    // [R][K]
  uint32_t* status;
  uint64_t d, seed;
  uint32_t L, K, NWT, NSEL, NCB, NWC, QB, nfast, nbig, s, w_idx, w_lev, w_val, sparsifier, quantizer, cap_words;
};

__device__ __forceinline__ uint32_t key_of_value(uint32_t vbits) { return (vbits & 0x7FFFFFFFu) << 1; }

// quantiser families: QSGD and its scaled form (Lemma 2) share everything but the transmitted norm
__host__ __device__ __forceinline__ bool is_qsgd(uint32_t q) { return q == QSL_QSGD || q == QSL_QSGD_SCALED; }
// which exact sum the quantiser's scale needs: squares (l2 norm), magnitudes (l1 norm), none
__host__ __device__ __forceinline__ bool wants_squares(uint32_t q) { return is_qsgd(q) || q == QSL_SIGN_L2; }

__device__ __forceinline__ uint32_t eff_path(const UnitState& us) {
  return us.path == PATH_FAST && us.fell_back ? static_cast<uint32_t>(PATH_FALLBACK) : us.path;
}

// Find, scanning the first NBINS bins of a histogram from the top, the bin in which the running count
// reaches `target` (1-based).  NT threads (the whole block), thread t owns the NBINS/NT bins below
// NBINS - t * NBINS/NT.  Returns the bin; *above = count in the bins above it.  If the histogram
// holds fewer than `target` entries, returns bin 0 with *above = total - hist[0].  If `clear`,
// zeroes the histogram afterwards.
template <uint32_t NT, uint32_t NBINS = HBINS>
__device__ uint32_t find_from_top(uint32_t* hist, uint32_t target, uint32_t* above, uint64_t* scratch,
                                  uint32_t* result, bool clear) {
  constexpr uint32_t PER = NBINS / NT;
  static_assert(PER >= 1 && PER * NT == NBINS, "bins must divide evenly over the threads");
  const uint32_t t = threadIdx.x;
  uint32_t h[PER]; uint32_t sum = 0;
#pragma unroll
  for (uint32_t j = 0; j < PER; ++j) { h[j] = hist[NBINS - 1 - (PER * t + j)]; sum += h[j]; }
  uint64_t total;
  const uint64_t before = block_exclusive_scan64(sum, scratch, &total);
  if (t == NT - 1) { result[0] = 0; result[1] = static_cast<uint32_t>(total) - h[PER - 1]; }
  __syncthreads();
  if (before < target && before + sum >= target) {
    uint32_t cum = static_cast<uint32_t>(before);
#pragma unroll
    for (uint32_t j = 0; j < PER; ++j) {
      if (cum + h[j] >= target) { result[0] = NBINS - 1 - (PER * t + j); result[1] = cum; break; }
      cum += h[j];
    }
  }
  if (clear) {
#pragma unroll
    for (uint32_t j = 0; j < PER; ++j) if (h[j]) hist[NBINS - 1 - (PER * t + j)] = 0;
  }
  __syncthreads();
  *above = result[1];
  return result[0];
}

__device__ __forceinline__ void flush_hist(const uint32_t* lh, uint32_t* gh) {
  for (uint32_t i = threadIdx.x; i < HBINS; i += blockDim.x) {
    const uint32_t v = lh[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

// ------------------------------------------------------------------------------------------------
// one-time initialisation of the static part of the unit states (at qsl_create)
// ------------------------------------------------------------------------------------------------
__global__ void k_init(DevCtx c, uint32_t U) {
  const uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= U) return;
  const SegInfo& sg = c.segs[u % c.L];
  UnitState s;
  s.path = sg.mode; s.T = sg.mode == PATH_FAST ? sg.T_static : 0xFFFFFFFFu; s.cand = 0; s.fell_back = 0;
  s.prefix1 = 0; s.k_rem1 = sg.k; s.prefix2 = 0; s.k_rem2 = sg.k; s.tau = 0; s.need = 0; s.n_gt = 0; s.nnz = 0; s.scale_bits = 0; s.pad = 0;
  c.units[u] = s;
}

// ------------------------------------------------------------------------------------------------
// the guess for Top_k: histogram of the rank keys of a strided sample of v = m + Delta
// (runs of 64 consecutive coordinates, evenly spaced), then the key at a fixed rank of the sample.
// A unit too small for a sample to be reliable is read whole: the guess is then the lower edge of
// the histogram bin that holds the k-th largest of the maxima of groups of 16 coordinates, which
// can never lie above the k-th largest key.
// ------------------------------------------------------------------------------------------------
// With `xm` given, `delta` holds the local models and Delta = xm - delta is formed on the fly.
__global__ __launch_bounds__(BIG) void k_sample(DevCtx c, const float* m, const float* delta, const float* xm) {
  __shared__ uint32_t lh[HBINS];
  const SelInfo si = c.samps[blockIdx.x];
  const uint32_t seg = si.seg, w = blockIdx.y;
  const SegInfo sg = c.segs[seg];
  for (uint32_t i = threadIdx.x; i < HBINS; i += BIG) lh[i] = 0;
  __syncthreads();
  const uint64_t row = static_cast<uint64_t>(w) * c.d + sg.start;
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t nwaves = sg.nsamp * (BIG / 64);
  const uint64_t stride = sg.samp_stride;                // >= 64: the runs do not overlap
  if (stride == 64) {                                     // the whole unit: a wave per chunk, 16 values per lane
    for (uint64_t ch = si.j * (BIG / 64) + wave; ch < sg.nwt; ch += nwaves) {
      f4u a[4], b[4], x[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint64_t e = ch * CHUNK + t * 256 + lane * 4;
        a[t] = b[t] = x[t] = f4u{0.f, 0.f, 0.f, 0.f};
        if (e + 4 <= sg.size) {
          a[t] = *reinterpret_cast<const f4u*>(m + row + e);
          b[t] = *reinterpret_cast<const f4u*>(delta + row + e);
          if (xm != nullptr) x[t] = *reinterpret_cast<const f4u*>(xm + sg.start + e);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (e + j < sg.size) { a[t][j] = m[row + e + j]; b[t][j] = delta[row + e + j]; if (xm != nullptr) x[t][j] = xm[sg.start + e + j]; }
        }
      }
      // Only the largest key of each lane's 16 coordinates is counted: the k-th largest of these
      // group maxima cannot exceed the k-th largest key (k distinct coordinates are at least as large),
      // so the bin it falls in still gives a valid guess, for a sixteenth of the LDS atomics.
      uint32_t top = 0; bool any = false;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint64_t e = ch * CHUNK + t * 256 + lane * 4;
        if (xm != nullptr) b[t] = x[t] - b[t];
        const f4u vv = a[t] + b[t];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (e + j < sg.size) { top = max(top, key_of_value(__float_as_uint(vv[j]))); any = true; }
      }
      if (any) atomicAdd(&lh[top >> 20], 1u);
    }
  } else
  for (uint32_t run0 = si.j * (BIG / 64) + wave; run0 < sg.n_runs; run0 += 8 * nwaves) {     // 8 runs in flight
    float a[8], b[8]; bool ok[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint32_t run = run0 + r * nwaves;
      const uint64_t pos = static_cast<uint64_t>(run) * stride + lane;
      ok[r] = run < sg.n_runs && pos < sg.size;
      a[r] = ok[r] ? m[row + pos] : 0.f;
      b[r] = ok[r] ? delta[row + pos] : 0.f;
      if (xm != nullptr && ok[r]) b[r] = xm[sg.start + pos] - b[r];
    }
#pragma unroll
    for (int r = 0; r < 8; ++r)
      if (ok[r]) atomicAdd(&lh[key_of_value(__float_as_uint(a[r] + b[r])) >> 20], 1u);
  }
  __syncthreads();
  flush_hist(lh, c.hist + (static_cast<uint64_t>(w) * c.L + seg) * 3 * HBINS);
}

__global__ __launch_bounds__(BIG) void k_sample_scan(DevCtx c) {
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[2];
  const uint32_t seg = c.fast_segs[blockIdx.x], w = blockIdx.y;
  const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
  uint32_t above;
  const uint32_t bin = find_from_top<BIG>(c.hist + u * 3 * HBINS, c.segs[seg].r_s, &above, scratch, result, true);
  if (threadIdx.x == 0) c.units[u].T = bin << 20;      // the guess: lower edge of the bin
}

// ------------------------------------------------------------------------------------------------
// the streaming pass.  One wave per chunk of 1024 coordinates: 8 + 4 dwordx4 accesses with
// streaming (non-temporal) cache hints, then the chunk's candidates go to the chunk's slot.
//
// Slot of a chunk: lpc * 2 elements of 8 bytes.  Element 0 is the header (count, overflow offset);
// elements 1 .. count hold (coordinate, value bits) in coordinate order.  A chunk with more
// candidates than its slot holds puts all of them into the unit's overflow pool instead (one
// returning atomic; rare unless the large values cluster) and records where.
// ------------------------------------------------------------------------------------------------
struct StreamSeg { uint64_t start, size, slot_off, ovf_off; uint32_t lpc, ovf_cap; };

typedef uint32_t u2v __attribute__((ext_vector_type(2)));

// DIFF: `delta` holds the local models xhat_{t+1/2} and `xm` the master's model x_t (one row of d floats,
// shared by the workers); Delta = x_t - xhat_{t+1/2} (Algorithm 1, sync step) is formed in registers.  The
// grid is then one-dimensional and ordered so that the R blocks that read the same four chunks of x_t
// follow each other on the same XCD (blocks go to the 8 XCDs round-robin), whose L2 serves R - 1 of them.
// Occupancy is held to 3 waves per SIMD for a single-segment context (4 otherwise): measured on the
// 8 x 25.6 M pass, 8 waves per SIMD 417 us, 5: 404, 4: 398, 3: 390, 2: 411 -- more requests in flight than
// the memory system wants only make it slower; the segmented and the x_t-reading forms were best at 4.
template <int SPARS, bool SINGLE, bool DIFF>
__global__ __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(SINGLE && !DIFF ? 3 : 4, SINGLE && !DIFF ? 3 : 4))) void k_stream(DevCtx c, StreamSeg one, const float* m, const float* delta,
                                                  const float* xm, float* m_out, uint32_t worker0, uint64_t round,
                                                  uint32_t R) {
  __shared__ uint2 s_stage[BLOCK / 64][32];
  __shared__ uint32_t s_stage_key[SPARS == QSL_RANDK ? BLOCK / 64 : 1][32];
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  uint32_t blk = blockIdx.x, w = blockIdx.y;
  if (DIFF) {
    const uint32_t slot = blockIdx.x >> 3;
    w = slot % R;
    blk = (slot / R) * 8 + (blockIdx.x & 7u);
  }
  const uint32_t wt = blk * 4 + wave;
  if (wt >= c.NWT) return;
  StreamSeg sg = one;
  uint32_t seg = 0, chunk = wt;
  if (!SINGLE) {
    const WtInfo wi = c.wts[wt];
    const SegInfo& s = c.segs[wi.seg];
    seg = wi.seg; chunk = wi.chunk;
    sg.start = s.start; sg.size = s.size; sg.slot_off = s.slot_off; sg.ovf_off = s.ovf_off;
    sg.lpc = s.lpc; sg.ovf_cap = s.ovf_cap;
  }
  const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
  const uint32_t T = c.units[u].T;
  const uint32_t path = c.units[u].path;
  const uint64_t row = static_cast<uint64_t>(w) * c.d + sg.start;
  const float* mp = m + row;
  const float* dp = delta + row;
  const float* xp = DIFF ? xm + sg.start : nullptr;
  float* op = m_out + row;
  const uint64_t cb = static_cast<uint64_t>(chunk) * CHUNK;           // segment-local
  f4u v[4];
  if (sg.size - cb >= CHUNK) {
    f4u a[4], b[4], x[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint64_t e = cb + t * 256 + lane * 4;
      a[t] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(mp + e));
      b[t] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(dp + e));
      if (DIFF) x[t] = *reinterpret_cast<const f4u*>(xp + e);        // cached: the other workers read it too
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (DIFF) b[t] = x[t] - b[t];
      v[t] = a[t] + b[t];
      __builtin_nontemporal_store(v[t], reinterpret_cast<f4u*>(op + cb + t * 256 + lane * 4));
    }
  } else {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint64_t e = cb + t * 256 + lane * 4 + j;
        float x = 0.0f;                                               // past the end: never a candidate
        if (e < sg.size) {
          const float dl = DIFF ? xp[e] - dp[e] : dp[e];
          x = mp[e] + dl; op[e] = x;
        }
        v[t][j] = x;
      }
    }
  }
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  uint32_t pm = 0;                                                    // bit t*4+j: coordinate (t, j) is a candidate
  bool nonfinite = false;
  Words4 rws[4];                                                      // Rand_k: the keys, kept for the slot's key line
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    Words4 rw;
    if (SPARS == QSL_RANDK) { rw = rand_words4(rk, static_cast<uint32_t>(sg.start + cb + t * 256 + lane * 4)); rws[t] = rw; }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t bits = __float_as_uint(v[t][j]);
      nonfinite |= (bits & 0x7FFFFFFFu) >= 0x7F800000u;
      const uint32_t key = SPARS == QSL_TOPK ? key_of_value(bits) : rw.w[j];
      const bool inside = cb + t * 256 + lane * 4 + j < sg.size;
      pm |= (inside && key >= T ? 1u : 0u) << (t * 4 + j);
    }
  }
  if (__ballot(nonfinite) != 0 && lane == 0) atomicOr(c.status, 1u);
  if (path != PATH_FAST) return;                  // uniform over the wave

  const uint32_t cap = sg.lpc * 2 - 1;
  uint2* stage = s_stage[wave];
  uint32_t total = 0, ovf_at = 0;
  if (__ballot(pm != 0) != 0) {
    uint32_t before[4], tot[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      before[t] = 0; tot[t] = 0;
      const uint32_t nib = (pm >> (t * 4)) & 0xFu;
      if (__ballot(nib != 0) == 0) continue;      // wave-uniform
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint64_t bal = __ballot((nib >> j) & 1u);
        before[t] += popc_below(bal);
        tot[t] += __popcll(bal);
      }
    }
    total = tot[0] + tot[1] + tot[2] + tot[3];
    uint32_t* ctr = c.ctr + u * (CTR_LINES * PAD);
    uint2* dst = stage + 1;                       // where entry 0 goes
    uint32_t* dst_key = SPARS == QSL_RANDK ? s_stage_key[wave] + 1 : nullptr;
    bool write = true;
    if (total > cap) {                            // wave-uniform: the slot cannot hold this chunk
      if (lane == 0) {
        ovf_at = atomicAdd(&ctr[CTR_OVF * PAD], total);
        if (ovf_at > sg.ovf_cap || total > sg.ovf_cap - ovf_at) { atomicOr(&ctr[CTR_FAIL * PAD], 1u); ovf_at = 0xFFFFFFFFu; }
      }
      ovf_at = __shfl(ovf_at, 0, WAVE);
      write = ovf_at != 0xFFFFFFFFu;
      dst = c.ovf + static_cast<uint64_t>(w) * c.ovf_stride + sg.ovf_off + ovf_at;
      if (SPARS == QSL_RANDK) dst_key = c.ovf_key + static_cast<uint64_t>(w) * c.ovf_stride + sg.ovf_off + ovf_at;
    }
    if (lane == 0) atomicAdd(&ctr[(chunk & (NSUB - 1)) * PAD], total);          // nobody waits for this one
    if (write) {
      uint32_t base = 0;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint32_t nib = (pm >> (t * 4)) & 0xFu;
        uint32_t pos = base + before[t];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if ((nib >> j) & 1u) {
            if (SPARS == QSL_RANDK) dst_key[pos] = rws[t].w[j];
            dst[pos++] = make_uint2(static_cast<uint32_t>(sg.start + cb + t * 256 + lane * 4 + j), __float_as_uint(v[t][j]));
          }
        }
        base += tot[t];
      }
    }
  }
  if (lane == 0) stage[0] = make_uint2(total, ovf_at);
  // the staging line is private to the wave, whose lanes run in lockstep: order the LDS traffic only
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  if (lane < sg.lpc * 2) {
    const uint2 e = stage[lane];
    const u2v ev = {e.x, e.y};
    const uint64_t at = static_cast<uint64_t>(w) * c.slot_stride + sg.slot_off + static_cast<uint64_t>(chunk) * (sg.lpc * 2);
    __builtin_nontemporal_store(ev, reinterpret_cast<u2v*>(c.slots + at + lane));
    if (SPARS == QSL_RANDK) __builtin_nontemporal_store(s_stage_key[wave][lane], c.slot_key + at + lane);   // the slot's key line
  }
}

// ------------------------------------------------------------------------------------------------
// walking the candidates of a fast unit.  A wave reads 64 x 16 bytes of the slot area at a time,
// i.e. 64 / lpc whole slots; lane l holds elements 2 (l mod lpc) and 2 (l mod lpc) + 1 of its slot.
// ------------------------------------------------------------------------------------------------
struct SlotRow {
  uint32_t count;        // candidates of this lane's chunk (0 if the chunk does not exist)
  uint32_t ovf_at;       // where they are in the overflow pool, if count > cap
  uint32_t n;            // candidates this lane is responsible for: 0..2 of its own elements, or all
                         // `count` entries in the overflow pool if it holds the header of such a chunk
  bool spill;            // n entries are read from the overflow pool
  bool has0, has1;       // this lane's first / second element is a candidate
  uint32_t idx0, bits0, idx1, bits1;
  uint32_t key0, key1;   // Rand_k: their rank keys, from the slot's key line
};

__device__ __forceinline__ SlotRow read_slot_row(const uint2* slots, const uint32_t* slot_key, uint32_t lpc, uint32_t nwt,
                                                 uint64_t row, uint64_t nrows) {
  SlotRow r;
  const uint32_t lane = lane_id();
  const uint32_t sub = lane & (lpc - 1);
  uint4 q = make_uint4(0, 0, 0, 0);
  uint2 kq = make_uint2(0, 0);
  if (row < nrows && ((row * 64 + lane) >> (__ffs(lpc) - 1)) < nwt) {                                                 // lpc: 4, 8 or 16
    q = reinterpret_cast<const uint4*>(slots)[row * 64 + lane];
    if (slot_key) kq = reinterpret_cast<const uint2*>(slot_key)[row * 64 + lane];
  }
  r.key0 = kq.x; r.key1 = kq.y;
  const uint32_t leader = lane & ~(lpc - 1);
  r.count = __shfl(q.x, leader, WAVE);
  r.ovf_at = __shfl(q.y, leader, WAVE);
  const uint32_t cap = lpc * 2 - 1;
  const bool inl = r.count <= cap;
  const uint32_t e0 = sub * 2;                    // element numbers of this lane; element e holds candidate e - 1
  r.has0 = inl && e0 >= 1 && e0 <= r.count;
  r.has1 = inl && e0 + 1 <= r.count;
  r.spill = !inl && sub == 0;
  r.n = r.spill ? r.count : (r.has0 ? 1u : 0u) + (r.has1 ? 1u : 0u);
  r.idx0 = q.x; r.bits0 = q.y; r.idx1 = q.z; r.bits1 = q.w;
  return r;
}

__device__ __forceinline__ uint32_t wave_exclusive_scan32(uint32_t x, uint32_t* total) {
  uint32_t inc = x;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(inc, o, WAVE);
    if (lane_id() >= static_cast<uint32_t>(o)) inc += y;
  }
  *total = __shfl(inc, 63, WAVE);
  return inc - x;
}

// ------------------------------------------------------------------------------------------------
// radix selection, one kernel per digit
// ------------------------------------------------------------------------------------------------
template <int LEVEL>
__device__ __forceinline__ bool level_bin(uint32_t key, uint32_t prefix, uint32_t* bin) {
  if (LEVEL == 0) { *bin = key >> 20; return true; }
  if (LEVEL == 1) { *bin = (key >> 8) & 0xFFFu; return (key >> 20) == (prefix >> 20); }
  *bin = key & 0xFFu; return (key >> 8) == (prefix >> 8);
}

// Digit LEVEL of the k-th largest key.  The blocks of a unit build the digit's histogram (LDS, then
// a few global atomics per bin); which bin the previous digit fell in is recomputed by every block
// from the previous kernel's histogram.
//   fast unit, digit 0: reads the slot rows (every wave a contiguous range) and leaves the number of
//                       candidates each wave met;
//   fast unit, digit 1: reads them again and writes all candidates, in coordinate order, into the
//                       unit's dense list (the offset of a wave = sum of the earlier waves' counts);
//   fast unit, digit 2: reads the dense list;
//   general path:       reads v.
template <int LEVEL, int SPARS>
__global__ __launch_bounds__(BIG) void k_select(DevCtx c, SegInfo one, const float* v, uint32_t worker0, uint64_t round) {
  __shared__ uint32_t lh[HBINS];
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[2], s_ctr[CTR_LINES];
  // a single-segment context carries its plan in the kernel arguments: one dependent load less per block
  SelInfo si; si.seg = 0; si.j = blockIdx.x;
  if (c.L != 1) si = c.sels[blockIdx.x];
  const uint32_t w = blockIdx.y;
  const SegInfo sg = c.L == 1 ? one : c.segs[si.seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + si.seg;
  UnitState* usp = &c.units[u];
  const UnitState us = *usp;
  uint32_t* hist = c.hist + u * 3 * HBINS;
  for (uint32_t i = threadIdx.x; i < HBINS; i += BIG) lh[i] = 0;
  if (LEVEL == 0 && threadIdx.x < CTR_LINES)
    s_ctr[threadIdx.x] = sg.mode == PATH_FAST ? c.ctr[(u * CTR_LINES + threadIdx.x) * PAD] : 0u;
  __syncthreads();
  uint32_t path, prefix = 0, k_rem = sg.k;
  if (LEVEL == 0) {
    // a guess that produced too few candidates, or more than there is room for, is discarded here
    path = us.path;
    if (path == PATH_FAST) {
      uint32_t cand = 0;
      for (uint32_t i = 0; i < NSUB; ++i) cand += s_ctr[i];
      if (s_ctr[CTR_FAIL] || cand < sg.k || cand > sg.d0_cap) path = PATH_FALLBACK;
      if (threadIdx.x == 0 && si.j == 0) { usp->cand = cand; usp->fell_back = path == PATH_FALLBACK; }
    } else if (threadIdx.x == 0 && si.j == 0) { usp->cand = 0; usp->fell_back = 0; }
    if (threadIdx.x == 0 && si.j == 0) usp->nnz = 0;
  } else {
    path = eff_path(us);
    uint32_t above;
    if (LEVEL == 1) {
      const uint32_t bin = find_from_top<BIG>(hist, sg.k, &above, scratch, result, false);
      prefix = bin << 20; k_rem = sg.k - above;
    } else {
      const uint32_t bin = find_from_top<BIG>(hist + HBINS, us.k_rem1, &above, scratch, result, false);
      prefix = us.prefix1 | (bin << 8); k_rem = us.k_rem1 - above;
    }
    if (threadIdx.x == 0 && si.j == 0) {
      if (LEVEL == 1) { usp->prefix1 = prefix; usp->k_rem1 = k_rem; }
      else { usp->prefix2 = prefix; usp->k_rem2 = k_rem; }
    }
  }
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  if (path == PATH_FAST && LEVEL < 2) {
    const uint2* slots = c.slots + static_cast<uint64_t>(w) * c.slot_stride + sg.slot_off;
    const uint2* ovf = c.ovf + static_cast<uint64_t>(w) * c.ovf_stride + sg.ovf_off;
    const uint32_t* slot_key = SPARS == QSL_RANDK ? c.slot_key + static_cast<uint64_t>(w) * c.slot_stride + sg.slot_off : nullptr;
    const uint32_t* ovf_key = SPARS == QSL_RANDK ? c.ovf_key + static_cast<uint64_t>(w) * c.ovf_stride + sg.ovf_off : nullptr;
    uint2* d0 = c.d0 + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
    uint32_t* d0k = c.d0_key + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
    uint32_t* wcnt = c.wave_cnt + static_cast<uint64_t>(w) * c.NWC + sg.wc_base;
    const uint32_t nrows = static_cast<uint32_t>((static_cast<uint64_t>(sg.nwt) * sg.lpc + 63) >> 6);   // < 2^20
    const uint32_t nwaves = sg.nsel * (BIG / 64), gw = si.j * (BIG / 64) + wave;
    const uint32_t rpw = (nrows + nwaves - 1) / nwaves;
    const uint64_t r_lo = static_cast<uint64_t>(gw) * rpw, r_hi = r_lo + rpw < nrows ? r_lo + rpw : nrows;
    uint32_t seen = 0;                              // digit 0: candidates this wave met
    uint32_t off = 0;                               // digit 1: where this wave's candidates go in the dense list
    if (LEVEL == 1) {                               // at most MAX_SELECT_BLOCKS * 16 = 1024 waves: 16 loads in flight
      uint32_t part[MAX_SELECT_BLOCKS * (BIG / 64) / WAVE];
#pragma unroll
      for (uint32_t i = 0; i < MAX_SELECT_BLOCKS * (BIG / 64) / WAVE; ++i) {
        const uint32_t g = i * WAVE + lane;
        part[i] = g < gw ? wcnt[g] : 0u;
      }
      uint32_t x = 0;
#pragma unroll
      for (uint32_t i = 0; i < MAX_SELECT_BLOCKS * (BIG / 64) / WAVE; ++i) x += part[i];
      off = wave_sum(x);
    }
    for (uint64_t row0 = r_lo; row0 < r_hi; row0 += 4) {
      SlotRow rr[4];                               // four independent accesses in flight; rows past the end read as empty
#pragma unroll
      for (int b = 0; b < 4; ++b) rr[b] = read_slot_row(slots, slot_key, sg.lpc, sg.nwt, row0 + b, r_hi);
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const SlotRow& r = rr[b];
        uint32_t pos = 0, tot = 0;
        if (LEVEL == 0) seen += r.n;
        else { pos = off + wave_exclusive_scan32(r.n, &tot); off += tot; }
        if (!r.spill) {
          uint32_t bin;
          if (r.has0) {
            const uint32_t key = SPARS == QSL_TOPK ? key_of_value(r.bits0) : r.key0;
            if (level_bin<LEVEL>(key, prefix, &bin)) atomicAdd(&lh[bin], 1u);
            if (LEVEL == 1) { d0[pos] = make_uint2(r.idx0, r.bits0); if (SPARS == QSL_RANDK) d0k[pos] = key; ++pos; }
          }
          if (r.has1) {
            const uint32_t key = SPARS == QSL_TOPK ? key_of_value(r.bits1) : r.key1;
            if (level_bin<LEVEL>(key, prefix, &bin)) atomicAdd(&lh[bin], 1u);
            if (LEVEL == 1) { d0[pos] = make_uint2(r.idx1, r.bits1); if (SPARS == QSL_RANDK) d0k[pos] = key; }
          }
        } else {
          for (uint32_t e = 0; e < r.count; ++e) {
            const uint2 ent = ovf[r.ovf_at + e];
            const uint32_t key = SPARS == QSL_TOPK ? key_of_value(ent.y) : ovf_key[r.ovf_at + e];
            uint32_t bin;
            if (level_bin<LEVEL>(key, prefix, &bin)) atomicAdd(&lh[bin], 1u);
            if (LEVEL == 1) { d0[pos + e] = ent; if (SPARS == QSL_RANDK) d0k[pos + e] = key; }
          }
        }
      }
    }
    if (LEVEL == 0) { seen = wave_sum(seen); if (lane == 0) wcnt[gw] = seen; }
  } else if (path == PATH_FAST) {
    const uint2* d0 = c.d0 + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
    const uint32_t* d0k = c.d0_key + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
    for (uint32_t e = si.j * BIG + threadIdx.x; e < us.cand; e += sg.nsel * BIG) {
      const uint32_t key = SPARS == QSL_TOPK ? key_of_value(d0[e].y) : d0k[e];
      uint32_t bin;
      if (level_bin<LEVEL>(key, prefix, &bin)) atomicAdd(&lh[bin], 1u);
    }
  } else {
    const float* vp = v + static_cast<uint64_t>(w) * c.d + sg.start;
    const uint32_t nwaves = sg.nsel * (BIG / 64);
    // a wave takes two chunks per step, 32 values per lane in flight
    for (uint64_t ch = (si.j * (BIG / 64) + wave) * 2; ch < sg.nwt; ch += 2ull * nwaves) {
      f4u x[2][4];
      if (SPARS == QSL_TOPK) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const uint64_t e = (ch + h) * CHUNK + t * 256 + lane * 4;
            x[h][t] = f4u{0.f, 0.f, 0.f, 0.f};
            if (e + 4 <= sg.size) x[h][t] = *reinterpret_cast<const f4u*>(vp + e);
            else {
#pragma unroll
              for (int j = 0; j < 4; ++j) if (e + j < sg.size) x[h][t][j] = vp[e + j];
            }
          }
        }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint64_t e = (ch + h) * CHUNK + t * 256 + lane * 4;
          Words4 rw = {{0u, 0u, 0u, 0u}};
          if (SPARS == QSL_RANDK && e < sg.size) rw = rand_words4(rk, static_cast<uint32_t>(sg.start + e));
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t key = SPARS == QSL_TOPK ? key_of_value(__float_as_uint(x[h][t][j])) : rw.w[j];
            uint32_t bin;
            if (e + j < sg.size && level_bin<LEVEL>(key, prefix, &bin)) atomicAdd(&lh[bin], 1u);
          }
        }
      }
    }
  }
  __syncthreads();
  flush_hist(lh, hist + LEVEL * HBINS);
}

// ------------------------------------------------------------------------------------------------
// ordered compaction of the selected coordinates, with the exact norm of what is selected.
//
// A "compaction block" covers either a tile of 2048 entries of a fast unit's dense candidate list
// (each thread 8 consecutive entries), or, on the general path, a contiguous range of groups of 16
// chunks of v (a group at a time: each wave 4 chunks, a lane 16 coordinates of a chunk; one group per
// block while the unit has at most 256 groups).  k_tile_count leaves the number of selected
// coordinates of every block; k_tile_write sums the earlier blocks' numbers to know where it writes.
// A fast unit whose guess failed runs the general path with the blocks it has.
//
// Exact norms: every |v| (or v^2) is an integer multiple of 2^-149 (2^-298); its 32-bit digits are
// added into 64-bit counters; integer addition commutes, so any schedule gives the same sum.
// ------------------------------------------------------------------------------------------------
constexpr uint32_t DTILE = 2048;           // dense-list entries per compaction block
constexpr uint32_t GGROUP = 16;            // chunks per general-path group
constexpr uint32_t ACC_ROWS = 32;          // accumulator rows of a compaction block (8 per wave)

struct Thresh { uint32_t tau, need; };

// one chunk of v in registers: 16 coordinates per lane, as two 16-bit masks (key > tau, key == tau)
template <int SPARS>
__device__ __forceinline__ void load_chunk_masks(const float* vp, uint64_t cb, uint64_t size, uint64_t start,
                                                 const RandKey& rk, Thresh th, f4u* val, uint32_t* gmask,
                                                 uint32_t* qmask) {
  const uint32_t lane = lane_id();
  uint32_t gm = 0, qm = 0;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const uint64_t e = cb + t * 256 + lane * 4;
    f4u x = {0.f, 0.f, 0.f, 0.f};
    if (e + 4 <= size) x = *reinterpret_cast<const f4u*>(vp + e);
    else {
#pragma unroll
      for (int j = 0; j < 4; ++j) if (e + j < size) x[j] = vp[e + j];
    }
    val[t] = x;
    Words4 rw;
    if (SPARS == QSL_RANDK) rw = rand_words4(rk, static_cast<uint32_t>(start + e));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t key = SPARS == QSL_TOPK ? key_of_value(__float_as_uint(x[j])) : rw.w[j];
      const bool inside = e + j < size;
      gm |= (inside && key > th.tau ? 1u : 0u) << (t * 4 + j);
      qm |= (inside && key == th.tau ? 1u : 0u) << (t * 4 + j);
    }
  }
  *gmask = gm; *qmask = qm;
}

// digits of |v| (or v^2) into an accumulator row in LDS that a few lanes share (hence the atomics)
__device__ __forceinline__ void lds_add(uint64_t* p, uint64_t x) {
  atomicAdd(reinterpret_cast<unsigned long long*>(p), static_cast<unsigned long long>(x));
}
__device__ __forceinline__ void add_digits(uint64_t* mine, uint32_t bits, bool squares) {
  const uint32_t ab = bits & 0x7FFFFFFFu;
  const uint32_t ex = ab >> 23, frac = ab & 0x7FFFFFu;
  const uint32_t M = ex ? (frac | 0x800000u) : frac;       // |v| = M * 2^(max(ex,1) - 150)
  const uint32_t e1 = ex ? ex : 1u;
  if (M == 0) return;
  if (squares) {
    const uint64_t sq = static_cast<uint64_t>(M) * M;       // < 2^48;  v^2 = sq * 2^(2 e1 - 300)
    const uint32_t p = 2u * e1 - 2u;                        // bit position above 2^-298
    const uint32_t q = p >> 5, r = p & 31u;
    const uint64_t lo = sq << r;                            // low 64 bits of sq * 2^r  (r <= 30)
    const uint64_t hi = r ? (sq >> (64 - r)) : 0;
    lds_add(&mine[q], lo & 0xFFFFFFFFu); lds_add(&mine[q + 1], lo >> 32);
    if (hi) lds_add(&mine[q + 2], hi);
  } else {
    const uint32_t p = e1 - 1u;                             // bit position above 2^-149
    const uint32_t q = p >> 5, r = p & 31u;
    const uint64_t sh = static_cast<uint64_t>(M) << r;      // < 2^55
    lds_add(&mine[q], sh & 0xFFFFFFFFu);
    if (sh >> 32) lds_add(&mine[q + 1], sh >> 32);
  }
}

// the general-path groups [g_lo, g_hi) of one unit, by one 256-thread block.
// WRITE = false: returns (in *tot_gt, *tot_eq, valid in thread 0) how many coordinates of these groups have key > tau / == tau.
// WRITE = true: writes the selected ones, in coordinate order, starting at ranks (gt0, eq0).
template <int SPARS, bool WRITE>
__device__ void general_groups(const SegInfo& sg, const float* vp, const RandKey& rk, Thresh th,
                               uint32_t g_lo, uint32_t g_hi, uint32_t gt0, uint32_t eq0, uint32_t* oi, uint32_t* ov,
                               uint64_t* mine, bool squares, uint32_t* s_cnt /*[2][GGROUP + 1]*/,
                               uint32_t* tot_gt, uint32_t* tot_eq) {
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  uint32_t run_gt = gt0, run_eq = eq0;             // ranks at the start of the current group (all threads agree)
  for (uint32_t g = g_lo; g < g_hi; ++g) {
    f4u val[4][4]; uint32_t gm[4], qm[4];
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      const uint32_t lc = wave * 4 + q;            // chunk inside the group: a wave takes 4 consecutive ones
      const uint64_t chunk = static_cast<uint64_t>(g) * GGROUP + lc;
      gm[q] = 0; qm[q] = 0;
      if (chunk < sg.nwt) load_chunk_masks<SPARS>(vp, chunk * CHUNK, sg.size, sg.start, rk, th, val[q], &gm[q], &qm[q]);
      const uint32_t cg = wave_sum(__popc(gm[q])), cq = wave_sum(__popc(qm[q]));
      if (lane == 0) { s_cnt[lc] = cg; s_cnt[GGROUP + 1 + lc] = cq; }
    }
    __syncthreads();
    if (threadIdx.x == 0) {                        // exclusive prefix over the 16 chunks, on top of the running ranks
      uint32_t a = run_gt, b = run_eq;
      for (uint32_t i = 0; i < GGROUP; ++i) {
        const uint32_t x = s_cnt[i], y = s_cnt[GGROUP + 1 + i];
        s_cnt[i] = a; s_cnt[GGROUP + 1 + i] = b; a += x; b += y;
      }
      s_cnt[GGROUP] = a; s_cnt[2 * GGROUP + 1] = b;
    }
    __syncthreads();
    if (WRITE) {
#pragma unroll
      for (uint32_t q = 0; q < 4; ++q) {
        if (__ballot((gm[q] | qm[q]) != 0) == 0) continue;          // wave-uniform
        const uint32_t lc = wave * 4 + q;
        const uint64_t cb = (static_cast<uint64_t>(g) * GGROUP + lc) * CHUNK;
        uint32_t base_gt = s_cnt[lc], base_eq = s_cnt[GGROUP + 1 + lc];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint32_t gn = (gm[q] >> (t * 4)) & 0xFu, qn = (qm[q] >> (t * 4)) & 0xFu;
          if (__ballot((gn | qn) != 0) == 0) continue;              // wave-uniform
          uint32_t bg = 0, bq = 0, tg = 0, tq = 0;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint64_t b1 = __ballot((gn >> j) & 1u), b2 = __ballot((qn >> j) & 1u);
            bg += popc_below(b1); tg += __popcll(b1); bq += popc_below(b2); tq += __popcll(b2);
          }
          uint32_t my_gt = base_gt + bg, my_eq = base_eq + bq;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const bool is_gt = (gn >> j) & 1u, is_eq = (qn >> j) & 1u;
            if (is_gt || (is_eq && my_eq < th.need)) {
              const uint32_t pos = my_gt + min(my_eq, th.need);
              const uint32_t bits = __float_as_uint(val[q][t][j]);
              oi[pos] = static_cast<uint32_t>(sg.start + cb + t * 256 + lane * 4 + j); ov[pos] = bits;
              add_digits(mine, bits, squares);
            }
            my_gt += is_gt; my_eq += is_eq;
          }
          base_gt += tg; base_eq += tq;
        }
      }
    }
    run_gt = s_cnt[GGROUP]; run_eq = s_cnt[2 * GGROUP + 1];
    __syncthreads();                               // s_cnt is reused by the next group
  }
  *tot_gt = run_gt - gt0; *tot_eq = run_eq - eq0;
}

// the threshold key and the tie budget, from the histogram of the last digit
__device__ __forceinline__ Thresh last_digit(const DevCtx& c, uint64_t u, const UnitState& us, uint64_t* scratch,
                                             uint32_t* result) {
  uint32_t above;
  const uint32_t bin = find_from_top<BLOCK, 256>(c.hist + (u * 3 + 2) * HBINS, us.k_rem2, &above, scratch, result, false);
  Thresh th; th.tau = us.prefix2 | bin; th.need = us.k_rem2 - above;
  return th;
}

// range of general-path groups a compaction block takes (one group each while the unit has at most 256)
__device__ __forceinline__ void fallback_range(const SegInfo& sg, uint32_t b, uint32_t* g_lo, uint32_t* g_hi) {
  const uint64_t ngg = (static_cast<uint64_t>(sg.nwt) + GGROUP - 1) / GGROUP;
  *g_lo = static_cast<uint32_t>(ngg * b / sg.ncb); *g_hi = static_cast<uint32_t>(ngg * (b + 1) / sg.ncb);
}

// ------------------------------------------------------------------------------------------------
// small units (at most 4 chunks = 4096 coordinates): the whole selection by one block of 256 threads.
// Thread t keeps 16 consecutive coordinates in registers (Top_k: the bits of v; Rand_k: the random
// words), the three digit histograms live in LDS, and the block writes the selected coordinates in order
// together with the digits of their norm -- what k_select<0..2>, k_tile_count and k_tile_write do for a
// larger unit, without a launch in between.  (One CU retires ~64 lane-operations per cycle: a block
// needed 25 us for 16,384 coordinates and 50 us for 65,536, and the slowest block is the kernel's time,
// so the limit is low; segments above it take the guessing path, whose kernels run anyway.)
// ------------------------------------------------------------------------------------------------
template <int LEVEL, int SPARS>
__device__ __forceinline__ void small_hist(const uint32_t (&kv)[16], uint32_t n, uint32_t prefix, uint32_t* lh) {
  const uint32_t e0 = threadIdx.x * 16;
#pragma unroll
  for (uint32_t j = 0; j < 16; ++j) {
    const uint32_t key = SPARS == QSL_TOPK ? key_of_value(kv[j]) : kv[j];
    uint32_t bin;
    if (e0 + j < n && level_bin<LEVEL>(key, prefix, &bin)) atomicAdd(&lh[bin], 1u);
  }
}

template <int SPARS>
__global__ __launch_bounds__(BLOCK) void k_small(DevCtx c, const float* v, uint32_t worker0, uint64_t round) {
  __shared__ uint32_t lh[HBINS];
  __shared__ uint64_t acc[ACC_ROWS * (ACC_SLOTS + 1)];
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[2];
  const uint32_t seg = c.small_segs[blockIdx.x], w = blockIdx.y;
  const SegInfo sg = c.segs[seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
  const float* vp = v + static_cast<uint64_t>(w) * c.d + sg.start;
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t n = static_cast<uint32_t>(sg.size);                 // <= SMALL_CHUNKS * CHUNK = 16 * BLOCK
  const uint32_t e0 = threadIdx.x * 16;
  uint32_t kv[16];
#pragma unroll
  for (uint32_t q = 0; q < 4; ++q) {
    const uint32_t e = e0 + q * 4;
    if (SPARS == QSL_TOPK) {
      f4u x = {0.f, 0.f, 0.f, 0.f};
      if (e + 4 <= n) x = *reinterpret_cast<const f4u*>(vp + e);
      else {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) if (e + j < n) x[j] = vp[e + j];
      }
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) kv[q * 4 + j] = __float_as_uint(x[j]);
    } else {
      Words4 rw = {{0u, 0u, 0u, 0u}};
      if (e < n) rw = rand_words4(rk, static_cast<uint32_t>(sg.start) + e);
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) kv[q * 4 + j] = rw.w[j];
    }
  }
  for (uint32_t i = threadIdx.x; i < ACC_ROWS * (ACC_SLOTS + 1); i += BLOCK) acc[i] = 0;

  // the three digits of the k-th largest key
  uint32_t above;
  for (uint32_t i = threadIdx.x; i < HBINS; i += BLOCK) lh[i] = 0;
  __syncthreads();
  small_hist<0, SPARS>(kv, n, 0, lh);
  __syncthreads();
  uint32_t bin = find_from_top<BLOCK>(lh, sg.k, &above, scratch, result, true);
  uint32_t prefix = bin << 20, k_rem = sg.k - above;
  small_hist<1, SPARS>(kv, n, prefix, lh);
  __syncthreads();
  bin = find_from_top<BLOCK>(lh, k_rem, &above, scratch, result, true);
  prefix |= bin << 8; k_rem -= above;
  small_hist<2, SPARS>(kv, n, prefix, lh);
  __syncthreads();
  bin = find_from_top<BLOCK, 256>(lh, k_rem, &above, scratch, result, false);
  const uint32_t tau = prefix | bin, need = k_rem - above;

  // ordered compaction: key > tau, and the first `need` coordinates with key == tau
  uint32_t gm = 0, qm = 0;
#pragma unroll
  for (uint32_t j = 0; j < 16; ++j) {
    const uint32_t key = SPARS == QSL_TOPK ? key_of_value(kv[j]) : kv[j];
    const bool inside = e0 + j < n;
    gm |= (inside && key > tau ? 1u : 0u) << j;
    qm |= (inside && key == tau ? 1u : 0u) << j;
  }
  uint64_t total;
  const uint64_t ex = block_exclusive_scan64((static_cast<uint64_t>(__popc(qm)) << 32) | __popc(gm), scratch, &total);
  const uint32_t gt0 = static_cast<uint32_t>(ex), eq0 = static_cast<uint32_t>(ex >> 32);
  // which of this thread's ties are kept: the first need - eq0 of them
  uint32_t keep = 0;
  if (eq0 < need) {
    keep = qm;
    for (uint32_t extra = eq0 + __popc(qm); extra > need; --extra) keep &= ~(0x80000000u >> __clz(keep));   // drop the last
  }
  const uint32_t sel = gm | keep;
  uint32_t* oi = c.sel_idx + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint32_t* ov = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint64_t* mine = acc + (wave * 8 + (lane & 7u)) * (ACC_SLOTS + 1);
  const bool squares = wants_squares(c.quantizer);
#pragma unroll
  for (uint32_t j = 0; j < 16; ++j) {
    if ((sel >> j) & 1u) {
      const uint32_t below = (1u << j) - 1u;
      const uint32_t pos = gt0 + __popc(gm & below) + min(eq0 + __popc(qm & below), need);
      const uint32_t bits = SPARS == QSL_TOPK ? kv[j] : __float_as_uint(vp[e0 + j]);
      oi[pos] = static_cast<uint32_t>(sg.start) + e0 + j; ov[pos] = bits;
      add_digits(mine, bits, squares);
    }
  }
  __syncthreads();
  // the unit is this block's alone: its norm digits are stored, not added
  for (uint32_t sl = wave; sl < ACC_SLOTS; sl += BLOCK / 64) {
    uint64_t x = lane < ACC_ROWS ? acc[lane * (ACC_SLOTS + 1) + sl] : 0;
    x = wave_sum64(x);
    if (lane == 0) c.norm_acc[u * ACC_SLOTS + sl] = x;
  }
  if (threadIdx.x == 0) {
    UnitState* us = &c.units[u];
    us->cand = 0; us->fell_back = 0; us->prefix2 = tau & ~0xFFu; us->k_rem2 = k_rem;
    us->tau = tau; us->need = need; us->n_gt = sg.k - need; us->nnz = 0;
  }
}

template <int SPARS>
__global__ __launch_bounds__(BLOCK) void k_tile_count(DevCtx c, SegInfo one, const float* v, uint32_t worker0, uint64_t round) {
  __shared__ uint32_t s_cnt[2 * GGROUP + 2], s_red[8], result[2];
  __shared__ uint64_t scratch[17];
  CbInfo cb; cb.seg = 0; cb.b = blockIdx.x;
  if (c.L != 1) cb = c.cbs[blockIdx.x];
  const uint32_t w = blockIdx.y;
  const SegInfo sg = c.L == 1 ? one : c.segs[cb.seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + cb.seg;
  const UnitState us = c.units[u];
  const uint32_t path = eff_path(us);
  if (path == PATH_FAST && cb.b != 0 && cb.b * DTILE >= us.cand) {         // a tile past the end of the dense list
    if (threadIdx.x == 0) c.cb_cnt[static_cast<uint64_t>(w) * c.NCB + sg.cb_base + cb.b] = make_uint2(0, 0);
    return;
  }
  const Thresh th = last_digit(c, u, us, scratch, result);
  if (threadIdx.x == 0 && cb.b == 0) { c.units[u].tau = th.tau; c.units[u].need = th.need; c.units[u].n_gt = sg.k - th.need; }
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  uint2* out = c.cb_cnt + static_cast<uint64_t>(w) * c.NCB + sg.cb_base + cb.b;
  if (path == PATH_FAST) {
    const uint2* d0 = c.d0 + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
    const uint32_t* d0k = c.d0_key + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
    uint32_t gt = 0, eq = 0;
    const uint32_t e0 = cb.b * DTILE + threadIdx.x * 8;
#pragma unroll
    for (uint32_t i = 0; i < 8; ++i) {
      if (e0 + i < us.cand) {
        const uint32_t key = SPARS == QSL_TOPK ? key_of_value(d0[e0 + i].y) : d0k[e0 + i];
        gt += key > th.tau; eq += key == th.tau;
      }
    }
    gt = wave_sum(gt); eq = wave_sum(eq);
    if (lane_id() == 0) { s_red[threadIdx.x >> 6] = gt; s_red[4 + (threadIdx.x >> 6)] = eq; }
    __syncthreads();
    if (threadIdx.x == 0) *out = make_uint2(s_red[0] + s_red[1] + s_red[2] + s_red[3], s_red[4] + s_red[5] + s_red[6] + s_red[7]);
    return;
  }
  uint32_t g_lo, g_hi;
  fallback_range(sg, cb.b, &g_lo, &g_hi);
  uint32_t tg = 0, tq = 0;
  general_groups<SPARS, false>(sg, v + static_cast<uint64_t>(w) * c.d + sg.start, rk, th, g_lo, g_hi, 0, 0, nullptr,
                               nullptr, nullptr, false, s_cnt, &tg, &tq);
  if (threadIdx.x == 0) *out = make_uint2(tg, tq);
}

template <int SPARS>
__global__ __launch_bounds__(BLOCK) void k_tile_write(DevCtx c, SegInfo one, const float* v, uint32_t worker0, uint64_t round) {
  __shared__ uint64_t acc[ACC_ROWS * (ACC_SLOTS + 1)];      // a row per 8 lanes of a wave: short atomic queues
  __shared__ uint32_t s_cnt[2 * GGROUP + 2];
  __shared__ uint64_t scratch[17], s_part[4];
  CbInfo cb; cb.seg = 0; cb.b = blockIdx.x;
  if (c.L != 1) cb = c.cbs[blockIdx.x];
  const uint32_t w = blockIdx.y;
  const SegInfo sg = c.L == 1 ? one : c.segs[cb.seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + cb.seg;
  const UnitState us = c.units[u];
  const uint32_t path = eff_path(us);
  if (path == PATH_FAST && cb.b * DTILE >= us.cand) return;                 // a tile past the end of the dense list
  Thresh th; th.tau = us.tau; th.need = us.need;
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const bool squares = wants_squares(c.quantizer);
  uint64_t* mine = acc + (wave * 8 + (lane & 7u)) * (ACC_SLOTS + 1);
  for (uint32_t i = threadIdx.x; i < ACC_ROWS * (ACC_SLOTS + 1); i += BLOCK) acc[i] = 0;   // published by the barrier below
  // how many selected coordinates precede this block: the sum of the unit's earlier blocks' counts
  {
    const uint2* cc = c.cb_cnt + static_cast<uint64_t>(w) * c.NCB + sg.cb_base;
    uint64_t x = 0;
    for (uint32_t i = threadIdx.x; i < cb.b; i += BLOCK) { const uint2 p = cc[i]; x += (static_cast<uint64_t>(p.y) << 32) | p.x; }
    x = wave_sum64(x);
    if (lane == 0) s_part[wave] = x;
  }
  __syncthreads();
  const uint64_t before = s_part[0] + s_part[1] + s_part[2] + s_part[3];
  const uint32_t gt0 = static_cast<uint32_t>(before), eq0 = static_cast<uint32_t>(before >> 32);
  uint32_t* oi = c.sel_idx + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint32_t* ov = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff;
  if (path == PATH_FAST) {
    const uint2* d0 = c.d0 + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
    const uint32_t* d0k = c.d0_key + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
    const uint32_t e0 = cb.b * DTILE + threadIdx.x * 8;
    uint2 ent[8]; uint32_t gm = 0, qm = 0;
#pragma unroll
    for (uint32_t i = 0; i < 8; ++i) {
      ent[i] = make_uint2(0, 0);
      if (e0 + i < us.cand) {
        ent[i] = d0[e0 + i];
        const uint32_t key = SPARS == QSL_TOPK ? key_of_value(ent[i].y) : d0k[e0 + i];
        gm |= (key > th.tau ? 1u : 0u) << i; qm |= (key == th.tau ? 1u : 0u) << i;
      }
    }
    uint64_t total;
    const uint64_t ex = block_exclusive_scan64((static_cast<uint64_t>(__popc(qm)) << 32) | __popc(gm), scratch, &total);
    uint32_t my_gt = gt0 + static_cast<uint32_t>(ex), my_eq = eq0 + static_cast<uint32_t>(ex >> 32);
#pragma unroll
    for (uint32_t i = 0; i < 8; ++i) {
      const bool is_gt = (gm >> i) & 1u, is_eq = (qm >> i) & 1u;
      if (is_gt || (is_eq && my_eq < th.need)) {
        const uint32_t pos = my_gt + min(my_eq, th.need);
        oi[pos] = ent[i].x; ov[pos] = ent[i].y;
        add_digits(mine, ent[i].y, squares);
      }
      my_gt += is_gt; my_eq += is_eq;
    }
  } else {
    uint32_t g_lo, g_hi;
    fallback_range(sg, cb.b, &g_lo, &g_hi);
    uint32_t tg, tq;
    general_groups<SPARS, true>(sg, v + static_cast<uint64_t>(w) * c.d + sg.start, rk, th, g_lo, g_hi, gt0, eq0, oi, ov,
                                mine, squares, s_cnt, &tg, &tq);
  }
  __syncthreads();
  uint64_t* ga = c.norm_acc + u * ACC_SLOTS;
  for (uint32_t s = wave; s < ACC_SLOTS; s += 4) {
    uint64_t x = lane < ACC_ROWS ? acc[lane * (ACC_SLOTS + 1) + s] : 0;
    x = wave_sum64(x);
    if (lane == 0 && x) atomicAdd(reinterpret_cast<unsigned long long*>(ga + s), static_cast<unsigned long long>(x));
  }
}

// digits -> one correctly rounded double -> the fp32 scale of the unit.  Called by all 64 lanes of a
// wave with the same arguments; lane i holds digit counter i, everything else is shuffles and ballots
// (a per-thread digit array would live in scratch memory and cost microseconds).
__device__ float finalize_scale(const uint64_t* acc, uint32_t quantizer, uint32_t k) {
  const bool squares = wants_squares(quantizer);
  const uint32_t lane = lane_id();
  const uint64_t a = lane < ACC_SLOTS ? acc[lane] : 0;
  // 32-bit digits: low half of the own counter plus the high half of the one below, then ripple the carries
  auto from_below = [&](uint32_t x) { const uint32_t y = __shfl_up(x, 1, WAVE); return lane ? y : 0u; };
  uint64_t t = (a & 0xFFFFFFFFull) + from_below(static_cast<uint32_t>(a >> 32));
  for (uint32_t it = 0; it < WAVE; ++it) {                            // ends after a few rounds; bounded anyway
    const uint32_t carry = static_cast<uint32_t>(t >> 32);
    if (__ballot(carry != 0) == 0) break;
    t = (t & 0xFFFFFFFFull) + from_below(carry);
  }
  const uint32_t dig = static_cast<uint32_t>(t);                      // digit `lane` of the exact sum
  const uint64_t nz = __ballot(dig != 0);
  double S = 0.0;
  if (nz != 0) {
    const int tw = 63 - __clzll(static_cast<long long>(nz));
    const int top = tw * 32 + 31 - __clz(static_cast<int>(__shfl(dig, tw, WAVE)));
    const int low = top - 52;                       // position of the last kept bit
    uint64_t mant; int e2;
    if (low <= 0) {
      mant = (static_cast<uint64_t>(__shfl(dig, 1, WAVE)) << 32) | __shfl(dig, 0, WAVE); e2 = 0;   // the whole value, exact
    } else {
      const int wq = low >> 5, r = low & 31;
      const uint64_t lo64 = (static_cast<uint64_t>(__shfl(dig, wq + 1, WAVE)) << 32) | __shfl(dig, wq, WAVE);
      const uint64_t hi32 = __shfl(dig, wq + 2, WAVE);                // lanes above the top digit hold 0
      uint64_t win = lo64 >> r;
      if (r) win |= hi32 << (64 - r);
      mant = win & ((1ull << 53) - 1);
      const int g = low - 1, gq = g >> 5, gb = g & 31;
      const uint32_t dg = __shfl(dig, gq, WAVE);
      const uint32_t guard = (dg >> gb) & 1u;
      const bool sticky = (dg & ((1u << gb) - 1u)) != 0 || __ballot(dig != 0 && lane < static_cast<uint32_t>(gq)) != 0;
      if (guard && (sticky || (mant & 1u))) mant += 1;
      e2 = low;
    }
    S = ldexp(static_cast<double>(mant), e2 + (squares ? -298 : -149));
  }
  if (quantizer == QSL_SIGN_L1) return static_cast<float>(S / static_cast<double>(k));           // ||v_S||_1 / k
  if (quantizer == QSL_SIGN_L2) return static_cast<float>(sqrt(S) / static_cast<double>(k));     // ||v_S||_2 / k
  if (quantizer == QSL_FP32) return 0.0f;
  return static_cast<float>(sqrt(S));                                                            // ||v_S||_2
}

// ------------------------------------------------------------------------------------------------
// quantise, error update, message
// ------------------------------------------------------------------------------------------------
// segment owning slot j of [K]: slot_dir[b] is the segment of slot b * 256 (same idea as seg_dir below)
__device__ __forceinline__ uint32_t seg_of_slot(const DevCtx& c, uint32_t j) {
  const uint32_t b = j >> 8;
  uint32_t lo = c.slot_dir[b], hi = c.slot_dir[b + 1] + 1;
  while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (c.segs[mid].koff <= j) lo = mid; else hi = mid; }
  return lo;
}
// segment of coordinate i: seg_dir[t] is the segment of coordinate t * 1024, so the search is over the few
// segments that touch one 1024-block instead of all L
__device__ __forceinline__ uint32_t seg_of_coord(const DevCtx& c, uint32_t i) {
  const uint32_t t = i >> 10;
  uint32_t lo = c.seg_dir[t], hi = c.seg_dir[t + 1] + 1;       // segs[lo].start <= i < segs[hi].start (or hi = L)
  while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (c.segs[mid].start <= i) lo = mid; else hi = mid; }
  return lo;
}

__device__ __forceinline__ float qsgd_value(float N, uint32_t level, uint32_t s, bool neg) {
  const float prod = N * static_cast<float>(level);
  const float mag = prod / static_cast<float>(s);
  return neg ? -mag : mag;
}

__global__ __launch_bounds__(BLOCK) void k_quantize(DevCtx c, float* m_out, uint32_t worker0, uint64_t round,
                                                    uint32_t* dbg_idx, uint16_t* dbg_level) {
  __shared__ uint32_t s_w[BLOCK / 64];
  __shared__ float s_scale[BLOCK], s_sent[BLOCK];
  const uint32_t w = blockIdx.y;
  const uint32_t j = blockIdx.x * BLOCK + threadIdx.x;
  // the scales of the units this block's slots belong to (at most one unit per slot)
  const uint32_t j_first = blockIdx.x * BLOCK, j_last = min(j_first + BLOCK, c.K) - 1;
  const uint32_t seg_first = c.L == 1 ? 0u : seg_of_slot(c, j_first);
  const uint32_t seg_last = c.L == 1 ? 0u : seg_of_slot(c, j_last);
  for (uint32_t i = threadIdx.x >> 6; i <= seg_last - seg_first; i += BLOCK / 64) {     // a wave per unit
    const uint32_t seg = seg_first + i;
    const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
    const uint32_t kl = c.segs[seg].k;
    const float sc = finalize_scale(c.norm_acc + u * ACC_SLOTS, c.quantizer, kl);
    if (lane_id() == 0) {
      s_scale[i] = sc;
      // what the message carries: the scale itself, or N / (1 + beta_{k,s}) for the scaled composition (Lemma 2)
      float sent = sc;
      if (c.quantizer == QSL_QSGD_SCALED) {
        const double beta = fmin(static_cast<double>(kl) / (static_cast<double>(c.s) * c.s), sqrt(static_cast<double>(kl)) / c.s);
        sent = sc / static_cast<float>(1.0 + beta);
      }
      s_sent[i] = sent;
      if (c.segs[seg].koff >= j_first) c.units[u].scale_bits = __float_as_uint(sent);   // the block holding the unit's first slot
    }
  }
  __syncthreads();
  uint32_t sent = 0;
  if (j < c.K) {
    const uint32_t seg = c.L == 1 ? 0u : seg_of_slot(c, j);
    const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
    const uint64_t slot = static_cast<uint64_t>(w) * c.K + j;
    const uint32_t idx = c.sel_idx[slot], bits = c.sel_val[slot];
    const float scale = s_scale[seg - seg_first];
    const float v = __uint_as_float(bits);
    const bool neg = v < 0.0f;
    uint32_t level;
    float g;
    if (is_qsgd(c.quantizer)) {
      level = 0;
      if (scale > 0.0f) {
        const float a = fabsf(v) / scale;
        float t = a * static_cast<float>(c.s);
        if (t > static_cast<float>(c.s)) t = static_cast<float>(c.s);
        const float fl = floorf(t);
        const float frac = t - fl;
        const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 1);
        const float r01 = static_cast<float>(rand_word(rk, idx) >> 8) * 0x1p-24f;
        level = static_cast<uint32_t>(fl) + (r01 < frac ? 1u : 0u);
      }
      g = qsgd_value(s_sent[seg - seg_first], level, c.s, neg);
    } else if (c.quantizer == QSL_FP32) {
      level = 1;
      g = v;
    } else {
      level = 1;
      g = neg ? -scale : scale;
    }
    sent = level != 0;
    c.sel_code[slot] = level | (neg ? 0x80000000u : 0u);
    if (sent) {
      if (idx < c.d) m_out[static_cast<uint64_t>(w) * c.d + idx] = v - g;
      else atomicOr(c.status, 2u);                       // cannot happen: a selected slot was never written
      if (is_qsgd(c.quantizer) && c.L > 1) atomicAdd(&c.units[u].nnz, 1u);
    }
    if (dbg_idx) dbg_idx[slot] = idx;
    if (dbg_level) dbg_level[slot] = static_cast<uint16_t>(level);
  }
  const uint32_t wc = __popcll(__ballot(sent));
  if (lane_id() == 0) s_w[threadIdx.x >> 6] = wc;
  __syncthreads();
  uint32_t* cnt = c.blk_cnt + static_cast<uint64_t>(w) * c.QB;
  if (threadIdx.x == 0) cnt[blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

// sum of cnt[0 .. n), by the whole block
__device__ __forceinline__ uint32_t block_sum_u32(const uint32_t* cnt, uint32_t n, uint32_t* s_part) {
  uint32_t x = 0;
  for (uint32_t i = threadIdx.x; i < n; i += BLOCK) x += cnt[i];
  x = wave_sum(x);
  __syncthreads();
  if (lane_id() == 0) s_part[threadIdx.x >> 6] = x;
  __syncthreads();
  return s_part[0] + s_part[1] + s_part[2] + s_part[3];
}

// only for very large K: exclusive prefix (and total) of the per-block survivor counts, one block per worker
__global__ __launch_bounds__(1024) void k_surv_scan(DevCtx c) {
  __shared__ uint64_t scratch[17];
  const uint32_t* cnt = c.blk_cnt + static_cast<uint64_t>(blockIdx.x) * c.QB;
  uint32_t* pre = c.blk_pre + static_cast<uint64_t>(blockIdx.x) * (c.QB + 1);
  uint64_t carry = 0;
  for (uint32_t base = 0; base < c.QB; base += 1024) {
    const uint32_t i = base + threadIdx.x;
    const uint64_t x = i < c.QB ? cnt[i] : 0;
    uint64_t total;
    const uint64_t ex = block_exclusive_scan64(x, scratch, &total) + carry;
    if (i < c.QB) pre[i] = static_cast<uint32_t>(ex);
    carry += total;
  }
  if (threadIdx.x == 0) pre[c.QB] = static_cast<uint32_t>(carry);
}

__global__ __launch_bounds__(BLOCK) void k_surv_compact(DevCtx c) {
  __shared__ uint32_t s_w[BLOCK / 64], s_part[4];
  const uint32_t w = blockIdx.y;
  const uint32_t j = blockIdx.x * BLOCK + threadIdx.x;
  // survivors before this block: the sum of the earlier blocks' counts
  const uint32_t before = c.QB > MAX_QB_INLINE
                              ? c.blk_pre[static_cast<uint64_t>(w) * (c.QB + 1) + blockIdx.x]
                              : block_sum_u32(c.blk_cnt + static_cast<uint64_t>(w) * c.QB, blockIdx.x, s_part);
  uint32_t code = 0;
  const uint64_t slot = static_cast<uint64_t>(w) * c.K + j;
  if (j < c.K) code = c.sel_code[slot];
  const bool sent = (code & 0x7FFFFFFFu) != 0;
  const uint64_t bal = __ballot(sent);
  if (lane_id() == 0) s_w[threadIdx.x >> 6] = __popcll(bal);
  __syncthreads();
  uint32_t pos = before + popc_below(bal);
  for (uint32_t i = 0; i < (threadIdx.x >> 6); ++i) pos += s_w[i];
  if (sent) {
    const uint32_t level = code & 0x7FFFFFFFu, neg = code >> 31;
    c.surv_idx[static_cast<uint64_t>(w) * c.K + pos] = c.sel_idx[slot];
    c.surv_code[static_cast<uint64_t>(w) * c.K + pos] = is_qsgd(c.quantizer) ? ((level - 1u) | (neg << c.w_lev))
                                                        : c.quantizer == QSL_FP32 ? c.sel_val[slot] : neg;
  }
}

// one thread per 32-bit word of the message: it gathers the fields that overlap its word
__device__ __forceinline__ uint32_t gather_word(const uint32_t* arr, uint64_t n, uint32_t width, uint64_t word) {
  if (width == 0) return 0;
  const uint64_t b0 = word * 32;
  const uint64_t e_end = min(n, (b0 + 31) / width + 1);           // one past the last field that touches the word
  uint32_t out = 0;
  for (uint64_t e0 = b0 / width; e0 < e_end; e0 += 8) {           // 8 loads in flight (a 1-bit field: 32 per word)
    uint32_t f[8];
#pragma unroll
    for (uint32_t i = 0; i < 8; ++i) f[i] = e0 + i < e_end ? arr[e0 + i] : 0u;
#pragma unroll
    for (uint32_t i = 0; i < 8; ++i) {
      if (e0 + i >= e_end) break;
      const int64_t sh = static_cast<int64_t>((e0 + i) * width) - static_cast<int64_t>(b0);
      out |= sh >= 0 ? (f[i] << sh) : (f[i] >> (-sh));
    }
  }
  return out;
}

__global__ __launch_bounds__(BLOCK) void k_pack(DevCtx c, uint8_t* msg, uint64_t* msg_bits) {
  __shared__ uint32_t s_part[4];
  const uint32_t w = blockIdx.y;
  // this is the last kernel of a call: it also returns the shared scratch of this worker to all-zero
  {
    const uint64_t tid = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x, nth = static_cast<uint64_t>(gridDim.x) * BLOCK;
    // histograms: only the segments that have any (not the one-block ones), and of the third digit only its 256 bins
    constexpr uint32_t ZW = 2 * HBINS + 256;
    uint32_t* h = c.hist + static_cast<uint64_t>(w) * c.L * 3 * HBINS;
    for (uint64_t i = tid; i < static_cast<uint64_t>(c.nbig) * ZW; i += nth)
      h[static_cast<uint64_t>(c.big_segs[i / ZW]) * 3 * HBINS + i % ZW] = 0;
    uint32_t* ct = c.ctr + static_cast<uint64_t>(w) * c.L * CTR_LINES * PAD;                 // counters: the guessing segments only
    for (uint64_t i = tid; i < static_cast<uint64_t>(c.nfast) * CTR_LINES; i += nth)
      ct[(static_cast<uint64_t>(c.fast_segs[i / CTR_LINES]) * CTR_LINES + i % CTR_LINES) * PAD] = 0;
    uint64_t* na = c.norm_acc + static_cast<uint64_t>(w) * c.L * ACC_SLOTS;
    for (uint64_t i = tid; i < static_cast<uint64_t>(c.L) * ACC_SLOTS; i += nth) na[i] = 0;
  }
  const uint64_t nnz = c.QB > MAX_QB_INLINE ? c.blk_pre[static_cast<uint64_t>(w) * (c.QB + 1) + c.QB]
                                            : block_sum_u32(c.blk_cnt + static_cast<uint64_t>(w) * c.QB, c.QB, s_part);
  const uint64_t q = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x;
  if (q >= c.cap_words) return;
  const bool counts = is_qsgd(c.quantizer) && c.L > 1;
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L) + (counts ? c.L : 0);
  const uint64_t idx_words = (nnz * c.w_idx + 31) / 32, code_words = (nnz * c.w_val + 31) / 32;
  uint32_t word = 0;
  if (q == 0) word = static_cast<uint32_t>(nnz);
  else if (q < 1 + static_cast<uint64_t>(c.L)) word = c.units[static_cast<uint64_t>(w) * c.L + (q - 1)].scale_bits;
  else if (q < hdr) word = c.units[static_cast<uint64_t>(w) * c.L + (q - 1 - c.L)].nnz;
  else if (q < hdr + idx_words) word = gather_word(c.surv_idx + static_cast<uint64_t>(w) * c.K, nnz, c.w_idx, q - hdr);
  else if (q < hdr + idx_words + code_words)
    word = gather_word(c.surv_code + static_cast<uint64_t>(w) * c.K, nnz, c.w_val, q - hdr - idx_words);
  reinterpret_cast<uint32_t*>(msg + static_cast<uint64_t>(w) * c.cap_words * 4)[q] = word;
  if (q == 0 && msg_bits) msg_bits[w] = hdr * 32 + nnz * (c.w_idx + c.w_val);
}

// ------------------------------------------------------------------------------------------------
// reading messages: stand-alone error update, aggregation
// ------------------------------------------------------------------------------------------------
struct MsgView {
  const uint32_t* words; uint32_t nnz; uint64_t idx_bit0, code_bit0;
};
__device__ __forceinline__ MsgView view_msg(const DevCtx& c, const uint8_t* msg, uint32_t row) {
  MsgView v;
  v.words = reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(row) * c.cap_words * 4);
  v.nnz = min(v.words[0], c.K);                         // a well-formed message never holds more than K entries
  const bool counts = is_qsgd(c.quantizer) && c.L > 1;
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L) + (counts ? c.L : 0);
  v.idx_bit0 = hdr * 32;
  v.code_bit0 = (hdr + (static_cast<uint64_t>(v.nnz) * c.w_idx + 31) / 32) * 32;
  return v;
}
__device__ __forceinline__ uint32_t msg_index(const DevCtx& c, const MsgView& v, uint32_t j) {
  return get_bits(v.words, v.idx_bit0 + static_cast<uint64_t>(j) * c.w_idx, c.w_idx);
}
__device__ __forceinline__ float msg_value(const DevCtx& c, const MsgView& v, uint32_t j, uint32_t idx) {
  const uint32_t code = get_bits(v.words, v.code_bit0 + static_cast<uint64_t>(j) * c.w_val, c.w_val);
  const uint32_t seg = c.L == 1 ? 0u : seg_of_coord(c, idx);
  const float scale = __uint_as_float(v.words[1 + seg]);
  if (is_qsgd(c.quantizer)) {
    const uint32_t level = (code & ((1u << c.w_lev) - 1u)) + 1u;
    return qsgd_value(scale, level, c.s, (code >> c.w_lev) & 1u);
  }
  if (c.quantizer == QSL_FP32) return __uint_as_float(code);
  return code ? -scale : scale;
}
// position of coordinate idx in the message, or -1
__device__ __forceinline__ int64_t msg_find(const DevCtx& c, const MsgView& v, uint32_t idx) {
  if (v.nnz == c.d) return idx;                          // every coordinate is there (k = d): entry j is coordinate j
  uint32_t lo = 0, hi = v.nnz;
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    const uint32_t x = msg_index(c, v, mid);
    if (x == idx) return mid;
    if (x < idx) lo = mid + 1; else hi = mid;
  }
  return -1;
}

// m <- m + delta over the flat [R * d] arrays: the streaming recipe of k_stream (a wave per 1024 elements,
// non-temporal dwordx4 accesses, 3 waves per SIMD)
__global__ __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(3, 3))) void k_add_rows(float* m, const float* delta,
                                                                                              uint64_t n) {
  const uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * (BLOCK / 64) + (threadIdx.x >> 6);
  const uint64_t cb = chunk * CHUNK;
  if (cb >= n) return;
  const uint32_t lane = lane_id();
  if (n - cb >= CHUNK) {
    f4u a[4], b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      a[t] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(m + cb + t * 256 + lane * 4));
      b[t] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(delta + cb + t * 256 + lane * 4));
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) __builtin_nontemporal_store(a[t] + b[t], reinterpret_cast<f4u*>(m + cb + t * 256 + lane * 4));
  } else {
    for (uint64_t i = cb + lane; i < n; i += 64) m[i] = m[i] + delta[i];
  }
}

__global__ __launch_bounds__(BLOCK) void k_subtract_msg(DevCtx c, float* m, const uint8_t* msg) {
  const uint32_t w = blockIdx.y;
  const MsgView v = view_msg(c, msg, w);
  const uint32_t j = blockIdx.x * BLOCK + threadIdx.x;
  if (j >= v.nnz) return;
  const uint32_t idx = msg_index(c, v, j);
  if (idx >= c.d) { atomicOr(c.status, 4u); return; }   // malformed message
  float* p = m + static_cast<uint64_t>(w) * c.d + idx;
  *p = *p - msg_value(c, v, j, idx);
}

__global__ __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(3, 3))) void k_fill_zero(float* out, uint64_t n) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * BLOCK * 4;
  const f4u z = {0.f, 0.f, 0.f, 0.f};
  for (uint64_t i = (static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 4 <= n) __builtin_nontemporal_store(z, reinterpret_cast<f4u*>(out + i));
    else for (uint64_t j = i; j < n; ++j) out[j] = 0.f;
  }
}

struct RowList { uint32_t row[64]; };
constexpr uint32_t AGG_ENTRIES = 32;     // message entries per block; 8 threads look one entry up in parallel
constexpr uint32_t AGG_DIR_SHIFT = 10;   // a directory entry per 1024 coordinates
constexpr uint32_t AGG_DIR_MIN = 4096;   // messages expected to be at least this long get a directory

// Directory of a long message: dir[t] = number of entries whose coordinate lies below t * 1024, for
// t = 0 .. ndir - 1 (ndir = ceil(d / 1024) + 1, so dir[ndir - 1] = nnz).  Entry j fills the slots between
// its predecessor's 1024-block and its own; the last entry also fills the rest.  A lookup then needs
// dir[t], dir[t + 1] and a binary search over the few entries of one 1024-block instead of log2(nnz)
// dependent probes of the whole message.
__global__ __launch_bounds__(BLOCK) void k_msg_directory(DevCtx c, const uint8_t* msg, RowList rows, uint32_t* dir,
                                                         uint32_t ndir) {
  const uint32_t q = blockIdx.y;
  const MsgView v = view_msg(c, msg, rows.row[q]);
  uint32_t* mine = dir + static_cast<uint64_t>(q) * ndir;
  const uint32_t nth = gridDim.x * BLOCK, tid = blockIdx.x * BLOCK + threadIdx.x;
  if (v.nnz == 0) { for (uint32_t t = tid; t < ndir; t += nth) mine[t] = 0; return; }
  for (uint32_t j = tid; j < v.nnz; j += nth) {
    const uint32_t cur = min(msg_index(c, v, j) >> AGG_DIR_SHIFT, ndir - 2);           // clamp: a malformed index
    const uint32_t first = j ? min(msg_index(c, v, j - 1) >> AGG_DIR_SHIFT, ndir - 2) + 1 : 0u;
    for (uint32_t t = first; t <= cur; ++t) mine[t] = j;                // empty when the predecessor shares the block
    if (j == v.nnz - 1) for (uint32_t t = cur + 1; t < ndir; ++t) mine[t] = v.nnz;
  }
}

// position of coordinate idx in a message with a directory, or -1
__device__ __forceinline__ int64_t msg_find_dir(const DevCtx& c, const MsgView& v, const uint32_t* dir, uint32_t idx) {
  if (v.nnz == c.d) return idx;                          // every coordinate is there (k = d): entry j is coordinate j
  const uint32_t t = idx >> AGG_DIR_SHIFT;
  uint32_t lo = dir[t], hi = min(dir[t + 1], v.nnz);
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    const uint32_t x = msg_index(c, v, mid);
    if (x == idx) return mid;
    if (x < idx) lo = mid + 1; else hi = mid;
  }
  return -1;
}

// Entry j of the q-th listed message is served by 8 threads, which look its coordinate up in the
// other listed messages (binary search on the packed, ascending indices).  The coordinate is
// written by the earliest listed message that holds it -- one writer per coordinate, no atomics --
// and the values are added in list order, so the result does not depend on the schedule.
__global__ __launch_bounds__(BLOCK) void k_aggregate(DevCtx c, const uint8_t* msg, RowList rows, uint32_t R,
                                                     float scale, int accumulate, float* out, const uint32_t* dir,
                                                     uint32_t ndir) {
  __shared__ float s_val[AGG_ENTRIES][65];
  __shared__ unsigned long long s_has[AGG_ENTRIES];
  const uint32_t q = blockIdx.y;
  const uint32_t e = threadIdx.x >> 3, sub = threadIdx.x & 7u;
  const MsgView mine = view_msg(c, msg, rows.row[q]);
  // the grid is sized for a moderate message; a block walks the tiles of 32 entries that exist
  for (uint32_t tile = blockIdx.x; tile * AGG_ENTRIES < mine.nnz; tile += gridDim.x) {
    const uint32_t j = tile * AGG_ENTRIES + e;
    if (sub == 0) s_has[e] = 0;
    __syncthreads();
    uint32_t idx = 0xFFFFFFFFu;
    if (j < mine.nnz) {
      idx = msg_index(c, mine, j);
      if (idx >= c.d) { if (sub == 0) atomicOr(c.status, 4u); idx = 0xFFFFFFFFu; }   // malformed message
    }
    if (idx != 0xFFFFFFFFu) {
      unsigned long long has = 0;
      for (uint32_t p = sub; p < R; p += 8) {
        if (p == q) { s_val[e][p] = msg_value(c, mine, j, idx); has |= 1ull << p; continue; }
        const MsgView other = view_msg(c, msg, rows.row[p]);
        const int64_t pos = dir ? msg_find_dir(c, other, dir + static_cast<uint64_t>(p) * ndir, idx) : msg_find(c, other, idx);
        if (pos >= 0) { s_val[e][p] = msg_value(c, other, static_cast<uint32_t>(pos), idx); has |= 1ull << p; }
      }
      if (has) atomicOr(&s_has[e], has);
    }
    __syncthreads();
    if (sub == 0 && idx != 0xFFFFFFFFu) {
      const unsigned long long has = s_has[e];
      if (!(has & ((1ull << q) - 1ull))) {                // no earlier listed message owns this coordinate
        float acc = 0.0f;
        bool first = true;
        for (uint32_t p = q; p < R; ++p) {
          if (!((has >> p) & 1ull)) continue;
          acc = first ? s_val[e][p] : acc + s_val[e][p];
          first = false;
        }
        const float term = scale * acc;
        out[idx] = accumulate ? out[idx] + term : term;
      }
    }
    __syncthreads();                                       // s_val and s_has are reused by the next tile
  }
}

__global__ void k_read_nnz(DevCtx c, const uint8_t* msg, uint32_t R, uint32_t* out) {
  const uint32_t r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < R) out[r] = reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(r) * c.cap_words * 4)[0];
}

uint32_t bit_width_u64(uint64_t x) { uint32_t w = 0; while (x) { ++w; x >>= 1; } return w; }

}  // namespace

// ====================================================================================================
// host side
// ====================================================================================================
struct qsl_ctx {
  qsl_config cfg;
  std::vector<uint64_t> off;
  std::vector<uint32_t> k;
  std::vector<SegInfo> segs;
  hipStream_t stream;
  DevCtx dc;
  StreamSeg one;
  void* slab;                 // one allocation holding every scratch array
  uint32_t Rmax;
  uint32_t last_R;
  uint32_t nsmall;            // segments selected by one block each (k_small)
  uint32_t nnz_hint;          // entries a message is expected to hold at most (sizes the aggregation grid)
  uint32_t* agg_dir;          // [64][agg_ndir] directories of the listed messages (only if messages are expected to be long)
  uint32_t agg_ndir;
  uint32_t n_sampled;         // segments whose guess comes from k_sample
  uint32_t nsamp_blocks;      // blocks of the sampling kernel (per worker)
  size_t capacity;
  uint32_t* h_status;         // pinned
  uint32_t* d_nnz_tmp;
  int timing;
  std::vector<hipEvent_t> ev;
  size_t ev_used;
};

#define QSL_HIP(call)                              \
  do {                                             \
    if ((call) != hipSuccess) return QSL_ERR_DEVICE; \
  } while (0)

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

extern "C" const char* qsl_status_string(qsl_status st) {
  switch (st) {
    case QSL_OK: return "ok";
    case QSL_ERR_INVALID_ARG: return "invalid argument";
    case QSL_ERR_BUFFER_TOO_SMALL: return "buffer too small";
    case QSL_ERR_NONFINITE_INPUT: return "non-finite value in m + delta";
    case QSL_ERR_DEVICE: return "HIP error";
    case QSL_ERR_UNSUPPORTED: return "unsupported";
  }
  return "unknown";
}

// argument checks of an operator description; *K_out = sum of the k_l
static qsl_status check_config(const qsl_config* cfg, uint64_t* K_out) {
  if (!cfg || !cfg->seg_offset || !cfg->seg_k) return QSL_ERR_INVALID_ARG;
  const uint64_t d = cfg->d;
  const uint32_t L = cfg->num_segments;
  if (d == 0 || d >= (1ull << 32) || L == 0 || L > 16384) return QSL_ERR_INVALID_ARG;
  if (cfg->sparsifier > 1 || cfg->quantizer > 4) return QSL_ERR_INVALID_ARG;
  if (is_qsgd(cfg->quantizer) && (cfg->s == 0 || cfg->s > 32768)) return QSL_ERR_INVALID_ARG;
  if (cfg->seg_offset[0] != 0 || cfg->seg_offset[L] != d) return QSL_ERR_INVALID_ARG;
  uint64_t K64 = 0;
  for (uint32_t l = 0; l < L; ++l) {
    if (cfg->seg_offset[l + 1] <= cfg->seg_offset[l]) return QSL_ERR_INVALID_ARG;
    const uint64_t size = cfg->seg_offset[l + 1] - cfg->seg_offset[l];
    if (cfg->seg_k[l] == 0 || cfg->seg_k[l] > size) return QSL_ERR_INVALID_ARG;
    K64 += cfg->seg_k[l];
  }
  if (K64 >= (1ull << 32)) return QSL_ERR_INVALID_ARG;
  *K_out = K64;
  return QSL_OK;
}

extern "C" qsl_status qsl_bits_index_free(const qsl_config* cfg, uint64_t* bits) {
  uint64_t K = 0;
  if (!bits) return QSL_ERR_INVALID_ARG;
  const qsl_status st = check_config(cfg, &K);
  if (st != QSL_OK) return st;
  if (cfg->sparsifier != QSL_RANDK) return QSL_ERR_UNSUPPORTED;      // Top_k's support depends on the data
  const uint64_t w = cfg->quantizer == QSL_FP32 ? 32 : is_qsgd(cfg->quantizer) ? bit_width_u64(cfg->s) + 1 : 1;
  *bits = 32ull * cfg->num_segments + K * w;
  return QSL_OK;
}

extern "C" qsl_status qsl_create(qsl_ctx** out, const qsl_config* cfg, void* hip_stream) {
  uint64_t K64 = 0;
  if (!out) return QSL_ERR_INVALID_ARG;
  const qsl_status cfg_status = check_config(cfg, &K64);
  if (cfg_status != QSL_OK) return cfg_status;
  if (cfg->max_workers == 0 || cfg->max_workers > 1024) return QSL_ERR_INVALID_ARG;
  const uint64_t d = cfg->d;
  const uint32_t L = cfg->num_segments;

  qsl_ctx* ctx = new (std::nothrow) qsl_ctx();
  if (!ctx) return QSL_ERR_DEVICE;
  ctx->cfg = *cfg;
  ctx->off.assign(cfg->seg_offset, cfg->seg_offset + L + 1);
  ctx->k.assign(cfg->seg_k, cfg->seg_k + L);
  ctx->cfg.seg_offset = ctx->off.data();
  ctx->cfg.seg_k = ctx->k.data();
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  ctx->Rmax = cfg->max_workers;
  ctx->last_R = 0;
  ctx->timing = 0; ctx->ev_used = 0;
  ctx->slab = nullptr; ctx->h_status = nullptr;

  const uint32_t K = static_cast<uint32_t>(K64);
  const uint32_t s = is_qsgd(cfg->quantizer) ? cfg->s : 1;
  // QSGD drops the entries it rounds to level 0: a segment keeps sum_i min(1, s |v_i| / ||v||_2) <= s sqrt(k)
  // of its k entries on average (Definition 1, example 1, with Cauchy-Schwarz); the other quantisers send all k
  double hint = 0;
  for (uint32_t l = 0; l < L; ++l) {
    const double kl = cfg->seg_k[l];
    hint += is_qsgd(cfg->quantizer) ? std::min(kl, 1.25 * s * std::sqrt(kl)) : kl;
  }
  ctx->nnz_hint = static_cast<uint32_t>(std::min<double>(hint, K));
  const uint32_t w_idx = std::max(1u, bit_width_u64(d - 1));
  const uint32_t w_lev = is_qsgd(cfg->quantizer) ? bit_width_u64(static_cast<uint64_t>(s) - 1) : 0;
  const uint32_t w_val = cfg->quantizer == QSL_FP32 ? 32 : w_lev + 1;
  const bool counts = is_qsgd(cfg->quantizer) && L > 1;
  uint64_t bits = 32 + 32ull * L + (counts ? 32ull * L : 0);
  bits += align_up(static_cast<uint64_t>(K) * w_idx, 32) + align_up(static_cast<uint64_t>(K) * w_val, 32);
  ctx->capacity = static_cast<size_t>(align_up(bits, 64) / 8);

  // per-segment plan: single-pass guessing ("fast") where the unit is large and sparse enough
  std::vector<SegInfo>& segs = ctx->segs;
  segs.resize(L);
  std::vector<WtInfo> wts;
  std::vector<SelInfo> sels, samps;
  std::vector<CbInfo> cbs;
  std::vector<uint32_t> fast, smalls;
  uint64_t slot_elems = 0, ovf_entries = 0, d0_entries = 0, nwt64 = 0, nwc = 0;
  uint32_t koff = 0;
  ctx->n_sampled = 0;
  for (uint32_t l = 0; l < L; ++l) {
    SegInfo& sg = segs[l];
    memset(&sg, 0, sizeof sg);
    sg.start = ctx->off[l]; sg.size = ctx->off[l + 1] - ctx->off[l];
    sg.k = ctx->k[l]; sg.koff = koff; koff += sg.k;
    sg.nwt = static_cast<uint32_t>((sg.size + CHUNK - 1) / CHUNK);
    nwt64 += sg.nwt;
    if (L > 1) {
      for (uint32_t t = 0; t < sg.nwt; ++t) { WtInfo wi; wi.seg = l; wi.chunk = t; wi.pad0 = wi.pad1 = 0; wts.push_back(wi); }
    }
    sg.mode = (sg.nwt <= SMALL_CHUNKS && !(cfg->flags & QSL_FLAG_NO_SMALL_PATH)) ? PATH_SMALL : PATH_GENERAL;
    sg.T_static = 0xFFFFFFFFu;
    sg.lpc = 8;
    const double n = static_cast<double>(sg.size), p = static_cast<double>(sg.k) / n;
    double cand = 0, slack = 0;                     // expected number of candidates, room beyond 4x that
    if (!(cfg->flags & QSL_FLAG_NO_FAST_PATH) && sg.nwt > SMALL_CHUNKS) {
      if (cfg->sparsifier == QSL_TOPK && static_cast<uint64_t>(sg.k) * 64 <= sg.size) {
        // candidates ~ alpha k; the sample must hold enough of them for the guess to sit below the
        // true threshold with ~6.5 sigma: (alpha - 1) sqrt(n_s p) >= 6.5 sqrt(alpha)
        // (a small unit has a small k, so a generous alpha costs few candidates and saves most of the sample)
        const double alphas[10] = {1.5, 2.0, 3.0, 4.0, 6.0, 8.0, 12.0, 16.0, 24.0, 32.0};
        for (double frac : {1.0 / 16, 1.0 / 4}) {
          for (double alpha : alphas) {
            const double n_s = 42.25 * alpha / ((alpha - 1) * (alpha - 1) * p);
            if (n_s > n * frac) continue;
            sg.n_runs = static_cast<uint32_t>(std::ceil(n_s / 64.0));
            sg.samp_stride = static_cast<uint32_t>(sg.size / sg.n_runs);
            sg.r_s = static_cast<uint32_t>(std::ceil(alpha * (sg.n_runs * 64.0) * p));
            sg.nsamp = std::min(MAX_SAMPLE_BLOCKS, std::max(1u, (sg.n_runs + 127) / 128));   // 8 runs per wave, all in flight
            cand = alpha * sg.k;
            slack = alpha <= 4.0 ? 8192.0 : 2048.0;
            break;
          }
          if (cand != 0) break;
        }
        if (cand == 0) {
          // no sample of at most 1/4 of the unit is reliable: read all of it (k * 64 <= size, so there are
          // at least 4 k groups of 16); the candidates are the k largest, the few more down to the k-th
          // largest group maximum, and the rest of the histogram bin (1/8 of a binade) that falls in
          sg.n_runs = static_cast<uint32_t>((sg.size + 63) / 64);
          sg.samp_stride = 64;
          sg.r_s = sg.k;
          sg.nsamp = std::min(MAX_SAMPLE_BLOCKS, std::max(1u, (sg.nwt + 63) / 64));      // four chunks per wave
          cand = 2.0 * sg.k;
          slack = 2048.0;
        }
        sg.d0_cap = static_cast<uint32_t>(std::min<double>(n, 4.0 * cand + slack));
        sg.mode = PATH_FAST;
        ++ctx->n_sampled;
        for (uint32_t j = 0; j < sg.nsamp; ++j) { SelInfo si; si.seg = l; si.j = j; si.pad0 = si.pad1 = 0; samps.push_back(si); }
      } else if (cfg->sparsifier == QSL_RANDK && static_cast<uint64_t>(sg.k) * 16 <= sg.size) {
        // the keys are uniform 32-bit words: keep those above the (1 - q) quantile, q = p + 7 sigma
        const double q = p + 7.0 * std::sqrt(p * (1 - p) / n);
        if (q * CHUNK <= 14.0) {                  // at most ~14 candidates per chunk: they fit a two-line slot
          sg.T_static = static_cast<uint32_t>(std::floor(4294967296.0 * (1.0 - q)));
          cand = q * n;
          sg.d0_cap = static_cast<uint32_t>(std::min<double>(n, cand + 8.0 * std::sqrt(cand) + 1024.0));
          sg.mode = PATH_FAST;
        }
      }
    }
    if (sg.mode == PATH_FAST) {
      // the slot of a chunk (64, 128 or 256 bytes) holds the expected candidates with ~4 sigma to spare;
      // chunks that hold more (chance, or clustered large values) spill to an overflow pool that can
      // take every candidate
      const double per_chunk = cand / sg.nwt, need = per_chunk + 4.0 * std::sqrt(per_chunk);
      sg.lpc = need <= 7.0 ? 4 : need <= 15.0 ? 8 : 16;
      fast.push_back(l);
      sg.slot_off = slot_elems; slot_elems += static_cast<uint64_t>(sg.nwt) * sg.lpc * 2;
      sg.ovf_cap = sg.d0_cap;
      sg.ovf_off = ovf_entries; ovf_entries += sg.ovf_cap;
      sg.d0_off = d0_entries; d0_entries += sg.d0_cap;
      sg.ncb = (sg.d0_cap + DTILE - 1) / DTILE;
    } else if (sg.mode == PATH_SMALL) {
      smalls.push_back(l);
      sg.nsel = 0; sg.ncb = 0;
    } else {
      sg.nsel = std::min(MAX_SELECT_BLOCKS, std::max(1u, (sg.nwt + 31) / 32));   // two chunks per wave up to 2^21 coordinates
      // at most 256 compaction blocks per unit, each a contiguous range of groups: every block ends with up to 20
      // atomics on the unit's digit counters, and thousands of blocks on the same few lines serialise there
      sg.ncb = std::min<uint32_t>(256, (sg.nwt + GGROUP - 1) / GGROUP);
    }
  }
  // blocks of a fast unit in the selection kernels: ~3 slot rows per wave, and no more than one block
  // per compute unit in all (measured, 8 workers with 1560 rows each: 16 blocks per unit 12 us, 32 blocks
  // 9 us, 48 blocks 12.5 us)
  uint64_t fast_blocks = 0;
  for (uint32_t l : fast) {
    SegInfo& sg = segs[l];
    const uint64_t nrows = (static_cast<uint64_t>(sg.nwt) * sg.lpc + 63) / 64;
    sg.nsel = static_cast<uint32_t>(std::min<uint64_t>(MAX_SELECT_BLOCKS, std::max<uint64_t>(1, (nrows + 47) / 48)));
    fast_blocks += static_cast<uint64_t>(sg.nsel) * ctx->Rmax;
  }
  if (fast_blocks > 256)
    for (uint32_t l : fast) segs[l].nsel = static_cast<uint32_t>(std::max<uint64_t>(1, segs[l].nsel * 256ull / fast_blocks));
  for (uint32_t l = 0; l < L; ++l) {
    SegInfo& sg = segs[l];
    for (uint32_t j = 0; j < sg.nsel; ++j) { SelInfo si; si.seg = l; si.j = j; si.pad0 = si.pad1 = 0; sels.push_back(si); }
    sg.wc_base = static_cast<uint32_t>(nwc); nwc += sg.nsel * (BIG / 64);
    sg.cb_base = static_cast<uint32_t>(cbs.size());
    for (uint32_t b = 0; b < sg.ncb; ++b) { CbInfo ci; ci.seg = l; ci.b = b; ci.pad0 = ci.pad1 = 0; cbs.push_back(ci); }
  }
  ctx->nsamp_blocks = static_cast<uint32_t>(samps.size());
  const uint32_t NWT = static_cast<uint32_t>(nwt64);
  const uint32_t NSEL = static_cast<uint32_t>(sels.size()), NCB = static_cast<uint32_t>(cbs.size());
  const uint32_t NWC = static_cast<uint32_t>(nwc);
  const uint32_t QB = (K + BLOCK - 1) / BLOCK;
  const uint64_t R = ctx->Rmax, U = R * L;

  // one slab, carved; the part that must be zero between calls comes first
  uint64_t bytes = 0;
  auto carve = [&](uint64_t n) { const uint64_t o = bytes; bytes = align_up(bytes + n, 256); return o; };
  const uint64_t o_hist = carve(4ull * 3 * HBINS * U), o_ctr = carve(4ull * CTR_LINES * PAD * U);
  const uint64_t o_acc = carve(8ull * ACC_SLOTS * U), o_status = carve(8);
  const uint64_t zero_bytes = bytes;
  const uint64_t o_segs = carve(sizeof(SegInfo) * L), o_wts = carve(sizeof(WtInfo) * std::max<size_t>(1, wts.size()));
  const uint64_t o_sels = carve(sizeof(SelInfo) * NSEL), o_cbs = carve(sizeof(CbInfo) * NCB);
  const uint64_t o_samps = carve(sizeof(SelInfo) * samps.size());
  const uint64_t o_fast = carve(4ull * std::max<size_t>(1, fast.size()));
  const uint64_t o_small = carve(4ull * std::max<size_t>(1, smalls.size()));
  std::vector<uint32_t> bigs;
  for (uint32_t l = 0; l < L; ++l) if (segs[l].mode != PATH_SMALL) bigs.push_back(l);
  const uint64_t o_big = carve(4ull * std::max<size_t>(1, bigs.size()));
  std::vector<uint32_t> seg_dir(((d + 1023) >> 10) + 1);
  for (size_t t = 0, l = 0; t < seg_dir.size(); ++t) {
    const uint64_t coord = std::min<uint64_t>(static_cast<uint64_t>(t) << 10, d - 1);
    while (l + 1 < L && ctx->off[l + 1] <= coord) ++l;
    seg_dir[t] = static_cast<uint32_t>(l);
  }
  const uint64_t o_segdir = carve(4ull * seg_dir.size());
  std::vector<uint32_t> slot_dir(((K + 255) >> 8) + 1);
  for (size_t b = 0, l = 0; b < slot_dir.size(); ++b) {
    const uint64_t slot = std::min<uint64_t>(static_cast<uint64_t>(b) << 8, K - 1);
    while (l + 1 < L && segs[l + 1].koff <= slot) ++l;
    slot_dir[b] = static_cast<uint32_t>(l);
  }
  const uint64_t o_slotdir = carve(4ull * slot_dir.size());
  const uint64_t o_units = carve(sizeof(UnitState) * U);
  const uint64_t o_slots = carve(8ull * std::max<uint64_t>(2, slot_elems) * R);
  const uint64_t o_ovf = carve(8ull * std::max<uint64_t>(1, ovf_entries) * R);
  const bool randk = cfg->sparsifier == QSL_RANDK;
  const uint64_t o_skey = carve(randk ? 4ull * std::max<uint64_t>(2, slot_elems) * R : 4);
  const uint64_t o_okey = carve(randk ? 4ull * std::max<uint64_t>(1, ovf_entries) * R : 4);
  const uint64_t o_d0 = carve(8ull * std::max<uint64_t>(1, d0_entries) * R);
  const uint64_t o_d0k = carve(4ull * std::max<uint64_t>(1, d0_entries) * R);
  const uint64_t o_wc = carve(4ull * NWC * R), o_cbc = carve(8ull * NCB * R);
  const uint64_t o_si = carve(4ull * K * R), o_sv = carve(4ull * K * R), o_sc = carve(4ull * K * R);
  const uint64_t o_blk = carve(4ull * QB * R), o_pre = carve(4ull * (QB + 1) * R);
  const uint64_t o_vi = carve(4ull * K * R), o_vc = carve(4ull * K * R);
  const uint64_t o_tmp = carve(4ull * 1024);
  ctx->agg_ndir = static_cast<uint32_t>(((d + (1u << AGG_DIR_SHIFT) - 1) >> AGG_DIR_SHIFT) + 1);
  const bool want_dir = ctx->nnz_hint >= AGG_DIR_MIN;
  const uint64_t o_dir = carve(want_dir ? 4ull * 64 * ctx->agg_ndir : 4);
  if (hipMalloc(&ctx->slab, bytes) != hipSuccess) { delete ctx; return QSL_ERR_DEVICE; }
  char* base = static_cast<char*>(ctx->slab);
  bool ok = hipMemset(base, 0, zero_bytes) == hipSuccess;
  auto upload = [&](uint64_t o, const void* src, size_t n) {
    if (n) ok = ok && hipMemcpy(base + o, src, n, hipMemcpyHostToDevice) == hipSuccess;
  };
  upload(o_segs, segs.data(), sizeof(SegInfo) * L);
  upload(o_wts, wts.data(), sizeof(WtInfo) * wts.size());
  upload(o_sels, sels.data(), sizeof(SelInfo) * NSEL);
  upload(o_samps, samps.data(), sizeof(SelInfo) * samps.size());
  upload(o_cbs, cbs.data(), sizeof(CbInfo) * NCB);
  upload(o_fast, fast.data(), 4 * fast.size());
  upload(o_small, smalls.data(), 4 * smalls.size());
  upload(o_big, bigs.data(), 4 * bigs.size());
  upload(o_segdir, seg_dir.data(), 4 * seg_dir.size());
  upload(o_slotdir, slot_dir.data(), 4 * slot_dir.size());
  ok = ok && hipHostMalloc(reinterpret_cast<void**>(&ctx->h_status), 64, hipHostMallocDefault) == hipSuccess;
  ok = ok && hipDeviceSynchronize() == hipSuccess;
  if (!ok) { (void)hipFree(ctx->slab); delete ctx; return QSL_ERR_DEVICE; }

  DevCtx& c = ctx->dc;
  c.segs = reinterpret_cast<const SegInfo*>(base + o_segs);
  c.wts = reinterpret_cast<const WtInfo*>(base + o_wts);
  c.sels = reinterpret_cast<const SelInfo*>(base + o_sels);
  c.samps = reinterpret_cast<const SelInfo*>(base + o_samps);
  c.cbs = reinterpret_cast<const CbInfo*>(base + o_cbs);
  c.fast_segs = reinterpret_cast<const uint32_t*>(base + o_fast);
  c.small_segs = reinterpret_cast<const uint32_t*>(base + o_small);
  c.big_segs = reinterpret_cast<const uint32_t*>(base + o_big); c.nbig = static_cast<uint32_t>(bigs.size());
  c.seg_dir = reinterpret_cast<const uint32_t*>(base + o_segdir);
  c.slot_dir = reinterpret_cast<const uint32_t*>(base + o_slotdir);
  ctx->nsmall = static_cast<uint32_t>(smalls.size());
  c.units = reinterpret_cast<UnitState*>(base + o_units);
  c.slots = reinterpret_cast<uint2*>(base + o_slots); c.slot_stride = std::max<uint64_t>(2, slot_elems);
  c.ovf = reinterpret_cast<uint2*>(base + o_ovf); c.ovf_stride = std::max<uint64_t>(1, ovf_entries);
  c.slot_key = reinterpret_cast<uint32_t*>(base + o_skey); c.ovf_key = reinterpret_cast<uint32_t*>(base + o_okey);
  c.d0 = reinterpret_cast<uint2*>(base + o_d0); c.d0_key = reinterpret_cast<uint32_t*>(base + o_d0k);
  c.d0_stride = std::max<uint64_t>(1, d0_entries);
  c.wave_cnt = reinterpret_cast<uint32_t*>(base + o_wc); c.cb_cnt = reinterpret_cast<uint2*>(base + o_cbc);
  c.hist = reinterpret_cast<uint32_t*>(base + o_hist); c.ctr = reinterpret_cast<uint32_t*>(base + o_ctr);
  c.norm_acc = reinterpret_cast<uint64_t*>(base + o_acc);
  c.sel_idx = reinterpret_cast<uint32_t*>(base + o_si); c.sel_val = reinterpret_cast<uint32_t*>(base + o_sv);
  c.sel_code = reinterpret_cast<uint32_t*>(base + o_sc);
  c.blk_cnt = reinterpret_cast<uint32_t*>(base + o_blk); c.blk_pre = reinterpret_cast<uint32_t*>(base + o_pre);
  c.surv_idx = reinterpret_cast<uint32_t*>(base + o_vi); c.surv_code = reinterpret_cast<uint32_t*>(base + o_vc);
  c.status = reinterpret_cast<uint32_t*>(base + o_status);
  ctx->d_nnz_tmp = reinterpret_cast<uint32_t*>(base + o_tmp);
  ctx->agg_dir = want_dir ? reinterpret_cast<uint32_t*>(base + o_dir) : nullptr;
  c.d = d; c.seed = cfg->seed; c.L = L; c.K = K; c.NWT = NWT; c.NSEL = NSEL; c.NCB = NCB; c.NWC = NWC; c.QB = QB;
  c.nfast = static_cast<uint32_t>(fast.size()); c.s = s; c.w_idx = w_idx; c.w_lev = w_lev; c.w_val = w_val;
  c.sparsifier = cfg->sparsifier; c.quantizer = cfg->quantizer;
  c.cap_words = static_cast<uint32_t>(ctx->capacity / 4);
  ctx->one.start = 0; ctx->one.size = segs[0].size; ctx->one.slot_off = 0; ctx->one.ovf_off = 0;
  ctx->one.lpc = segs[0].lpc; ctx->one.ovf_cap = segs[0].ovf_cap;
  k_init<<<dim3(static_cast<uint32_t>((U + 255) / 256)), 256, 0, ctx->stream>>>(c, static_cast<uint32_t>(U));
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) {
    (void)hipFree(ctx->slab); (void)hipHostFree(ctx->h_status); delete ctx; return QSL_ERR_DEVICE;
  }
  *out = ctx;
  return QSL_OK;
}

extern "C" qsl_status qsl_destroy(qsl_ctx* ctx) {
  if (!ctx) return QSL_ERR_INVALID_ARG;
  (void)hipStreamSynchronize(ctx->stream);
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  if (ctx->slab) (void)hipFree(ctx->slab);
  if (ctx->h_status) (void)hipHostFree(ctx->h_status);
  delete ctx;
  return QSL_OK;
}

extern "C" qsl_status qsl_set_stream(qsl_ctx* ctx, void* hip_stream) {
  if (!ctx) return QSL_ERR_INVALID_ARG;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  return QSL_OK;
}

extern "C" size_t qsl_msg_capacity_bytes(const qsl_ctx* ctx) { return ctx ? ctx->capacity : 0; }

template <int SPARS>
static qsl_status launch_compress(qsl_ctx* ctx, const float* m, const float* delta, const float* xm, float* m_out,
                                  uint32_t worker0,
                                  uint32_t R, uint64_t round, uint8_t* msg, uint64_t* msg_bits, uint32_t* sel_idx,
                                  uint16_t* sel_level) {
  const DevCtx& c = ctx->dc;
  hipStream_t st = ctx->stream;
  if (SPARS == QSL_TOPK && ctx->n_sampled > 0) {
    k_sample<<<dim3(ctx->nsamp_blocks, R), BIG, 0, st>>>(c, m, delta, xm);
    k_sample_scan<<<dim3(c.nfast, R), BIG, 0, st>>>(c);
  }
  const bool timed = ctx->timing != 0;
  if (timed) {
    if (ctx->ev_used + 2 > ctx->ev.size()) {
      for (int i = 0; i < 2; ++i) { hipEvent_t e; QSL_HIP(hipEventCreate(&e)); ctx->ev.push_back(e); }
    }
    QSL_HIP(hipEventRecord(ctx->ev[ctx->ev_used], st));
  }
  const uint32_t nblk = (c.NWT + 3) / 4;
  if (xm == nullptr) {
    const dim3 sgrid(nblk, R);
    if (c.L == 1) k_stream<SPARS, true, false><<<sgrid, BLOCK, 0, st>>>(c, ctx->one, m, delta, xm, m_out, worker0, round, R);
    else k_stream<SPARS, false, false><<<sgrid, BLOCK, 0, st>>>(c, ctx->one, m, delta, xm, m_out, worker0, round, R);
  } else {
    const uint64_t nb = static_cast<uint64_t>((nblk + 7) / 8) * 8 * R;
    if (nb > 0x7FFFFFFFull) return QSL_ERR_UNSUPPORTED;
    const dim3 sgrid(static_cast<uint32_t>(nb));
    if (c.L == 1) k_stream<SPARS, true, true><<<sgrid, BLOCK, 0, st>>>(c, ctx->one, m, delta, xm, m_out, worker0, round, R);
    else k_stream<SPARS, false, true><<<sgrid, BLOCK, 0, st>>>(c, ctx->one, m, delta, xm, m_out, worker0, round, R);
  }
  if (timed) { QSL_HIP(hipEventRecord(ctx->ev[ctx->ev_used + 1], st)); ctx->ev_used += 2; }

  if (ctx->nsmall) k_small<SPARS><<<dim3(ctx->nsmall, R), BLOCK, 0, st>>>(c, m_out, worker0, round);
  if (c.NSEL) {                                    // units that take a launch per digit and two for the compaction
    k_select<0, SPARS><<<dim3(c.NSEL, R), BIG, 0, st>>>(c, ctx->segs[0], m_out, worker0, round);
    k_select<1, SPARS><<<dim3(c.NSEL, R), BIG, 0, st>>>(c, ctx->segs[0], m_out, worker0, round);
    k_select<2, SPARS><<<dim3(c.NSEL, R), BIG, 0, st>>>(c, ctx->segs[0], m_out, worker0, round);
    k_tile_count<SPARS><<<dim3(c.NCB, R), BLOCK, 0, st>>>(c, ctx->segs[0], m_out, worker0, round);
    k_tile_write<SPARS><<<dim3(c.NCB, R), BLOCK, 0, st>>>(c, ctx->segs[0], m_out, worker0, round);
  }
  k_quantize<<<dim3(c.QB, R), BLOCK, 0, st>>>(c, m_out, worker0, round, sel_idx, sel_level);
  if (c.QB > MAX_QB_INLINE) k_surv_scan<<<dim3(R), 1024, 0, st>>>(c);
  k_surv_compact<<<dim3(c.QB, R), BLOCK, 0, st>>>(c);
  k_pack<<<dim3((c.cap_words + BLOCK - 1) / BLOCK, R), BLOCK, 0, st>>>(c, msg, msg_bits);
  QSL_HIP(hipGetLastError());
  return QSL_OK;
}

static qsl_status compress_checked(qsl_ctx* ctx, const float* m, const float* delta, const float* xm, float* m_out,
                                   uint32_t worker0, uint32_t R, uint64_t round, uint8_t* msg, uint64_t* msg_bits,
                                   uint32_t* sel_idx, uint16_t* sel_level) {
  if (!ctx || !m || !delta || !m_out || !msg || R == 0 || R > ctx->Rmax || (round >> 62)) return QSL_ERR_INVALID_ARG;
  if (static_cast<uint64_t>(worker0) + R > (1ull << 32)) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(delta) | reinterpret_cast<uintptr_t>(m_out) |
       reinterpret_cast<uintptr_t>(xm) | reinterpret_cast<uintptr_t>(sel_idx)) & 3) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(msg) | reinterpret_cast<uintptr_t>(msg_bits)) & 7) return QSL_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(sel_level) & 1) return QSL_ERR_INVALID_ARG;
  ctx->last_R = R;
  if (ctx->cfg.sparsifier == QSL_TOPK)
    return launch_compress<QSL_TOPK>(ctx, m, delta, xm, m_out, worker0, R, round, msg, msg_bits, sel_idx, sel_level);
  return launch_compress<QSL_RANDK>(ctx, m, delta, xm, m_out, worker0, R, round, msg, msg_bits, sel_idx, sel_level);
}

extern "C" qsl_status qsl_compress(qsl_ctx* ctx, const float* m, const float* delta, float* m_out, uint32_t worker0,
                                   uint32_t R, uint64_t round, uint8_t* msg, uint64_t* msg_bits, uint32_t* sel_idx,
                                   uint16_t* sel_level) {
  return compress_checked(ctx, m, delta, nullptr, m_out, worker0, R, round, msg, msg_bits, sel_idx, sel_level);
}

extern "C" qsl_status qsl_compress_diff(qsl_ctx* ctx, const float* m, const float* x, const float* xhat_half,
                                        float* m_out, uint32_t worker0, uint32_t R, uint64_t round, uint8_t* msg,
                                        uint64_t* msg_bits, uint32_t* sel_idx, uint16_t* sel_level) {
  if (!x) return QSL_ERR_INVALID_ARG;
  return compress_checked(ctx, m, xhat_half, x, m_out, worker0, R, round, msg, msg_bits, sel_idx, sel_level);
}

extern "C" qsl_status qsl_error_update(qsl_ctx* ctx, float* m, const float* delta, const uint8_t* msg, uint32_t R) {
  if (!ctx || !m || !delta || !msg || R == 0 || R > ctx->Rmax) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(delta)) & 3) return QSL_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(msg) & 7) return QSL_ERR_INVALID_ARG;
  const DevCtx& c = ctx->dc;
  const uint64_t n = static_cast<uint64_t>(R) * c.d;
  const uint64_t blocks = (n + CHUNK * (BLOCK / 64) - 1) / (CHUNK * (BLOCK / 64));
  if (blocks > 0x7FFFFFFFull) return QSL_ERR_UNSUPPORTED;
  k_add_rows<<<dim3(static_cast<uint32_t>(blocks)), BLOCK, 0, ctx->stream>>>(m, delta, n);
  k_subtract_msg<<<dim3((c.K + BLOCK - 1) / BLOCK, R), BLOCK, 0, ctx->stream>>>(c, m, msg);
  QSL_HIP(hipGetLastError());
  return QSL_OK;
}

extern "C" qsl_status qsl_aggregate(qsl_ctx* ctx, const uint8_t* msg, const uint32_t* worker_list, uint32_t R,
                                    float scale, int accumulate, float* out) {
  if (!ctx || !msg || !out || R == 0 || R > 64) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(msg) & 7) || (reinterpret_cast<uintptr_t>(out) & 3)) return QSL_ERR_INVALID_ARG;
  const DevCtx& c = ctx->dc;
  RowList rows;
  for (uint32_t q = 0; q < 64; ++q) rows.row[q] = q < R ? (worker_list ? worker_list[q] : q) : 0;
  for (uint32_t q = 0; q < R; ++q)
    for (uint32_t p = 0; p < q; ++p)
      if (rows.row[p] == rows.row[q]) return QSL_ERR_INVALID_ARG;       // a message may be listed once
  if (!accumulate) {
    const uint32_t blocks = static_cast<uint32_t>(std::min<uint64_t>((c.d + BLOCK * 4 - 1) / (BLOCK * 4), 1u << 16));
    k_fill_zero<<<dim3(blocks), BLOCK, 0, ctx->stream>>>(out, c.d);
  }
  const uint32_t tiles = (c.K + AGG_ENTRIES - 1) / AGG_ENTRIES;
  const uint32_t agg_blocks = std::min(tiles, std::max(16u, (ctx->nnz_hint + AGG_ENTRIES - 1) / AGG_ENTRIES));
  uint32_t* dir = R > 1 ? ctx->agg_dir : nullptr;
  if (dir) k_msg_directory<<<dim3(std::min(2048u, (c.K + BLOCK - 1) / BLOCK), R), BLOCK, 0, ctx->stream>>>(c, msg, rows, dir, ctx->agg_ndir);
  k_aggregate<<<dim3(agg_blocks, R), BLOCK, 0, ctx->stream>>>(c, msg, rows, R, scale, accumulate, out, dir, ctx->agg_ndir);
  QSL_HIP(hipGetLastError());
  return QSL_OK;
}

extern "C" qsl_status qsl_bits_sent(qsl_ctx* ctx, const uint8_t* msg, uint32_t R, uint64_t* bits_host) {
  if (!ctx || !msg || !bits_host || R == 0 || R > 1024) return QSL_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(msg) & 7) return QSL_ERR_INVALID_ARG;
  const DevCtx& c = ctx->dc;
  k_read_nnz<<<dim3((R + 255) / 256), 256, 0, ctx->stream>>>(c, msg, R, ctx->d_nnz_tmp);
  std::vector<uint32_t> nnz(R);
  QSL_HIP(hipMemcpyAsync(nnz.data(), ctx->d_nnz_tmp, 4ull * R, hipMemcpyDeviceToHost, ctx->stream));
  QSL_HIP(hipStreamSynchronize(ctx->stream));
  const bool counts = is_qsgd(c.quantizer) && c.L > 1;
  const uint64_t hdr = 32 + 32ull * c.L + (counts ? 32ull * c.L : 0);
  for (uint32_t r = 0; r < R; ++r) bits_host[r] = hdr + static_cast<uint64_t>(nnz[r]) * (c.w_idx + c.w_val);
  return QSL_OK;
}

extern "C" qsl_status qsl_device_status(qsl_ctx* ctx) {
  if (!ctx) return QSL_ERR_INVALID_ARG;
  QSL_HIP(hipMemcpyAsync(ctx->h_status, ctx->dc.status, 4, hipMemcpyDeviceToHost, ctx->stream));
  QSL_HIP(hipMemsetAsync(ctx->dc.status, 0, 4, ctx->stream));
  QSL_HIP(hipStreamSynchronize(ctx->stream));
  if (ctx->h_status[0] & 6u) return QSL_ERR_DEVICE;      // internal inconsistency or malformed message
  return (ctx->h_status[0] & 1u) ? QSL_ERR_NONFINITE_INPUT : QSL_OK;
}

extern "C" qsl_status qsl_debug_units(qsl_ctx* ctx, uint32_t* out_host, uint32_t max_units, uint32_t* n_units) {
  if (!ctx || !out_host || !n_units) return QSL_ERR_INVALID_ARG;
  const uint32_t U = ctx->last_R * ctx->dc.L;
  if (U > max_units) return QSL_ERR_BUFFER_TOO_SMALL;
  std::vector<UnitState> us(U);
  if (U) QSL_HIP(hipMemcpyAsync(us.data(), ctx->dc.units, sizeof(UnitState) * U, hipMemcpyDeviceToHost, ctx->stream));
  QSL_HIP(hipStreamSynchronize(ctx->stream));
  for (uint32_t u = 0; u < U; ++u) {
    uint32_t* o = out_host + 8ull * u;
    o[0] = us[u].path == PATH_FAST && us[u].fell_back ? static_cast<uint32_t>(PATH_FALLBACK) : us[u].path;
    o[1] = us[u].cand; o[2] = us[u].tau; o[3] = us[u].n_gt; o[4] = us[u].need; o[5] = us[u].T;
    o[6] = us[u].scale_bits; o[7] = us[u].nnz;
  }
  *n_units = U;
  return QSL_OK;
}

extern "C" qsl_status qsl_timing_enable(qsl_ctx* ctx, int enabled) {
  if (!ctx) return QSL_ERR_INVALID_ARG;
  ctx->timing = enabled; ctx->ev_used = 0;
  return QSL_OK;
}

extern "C" qsl_status qsl_timing_read(qsl_ctx* ctx, double* total_ms, uint32_t* launches) {
  if (!ctx || !total_ms || !launches) return QSL_ERR_INVALID_ARG;
  QSL_HIP(hipStreamSynchronize(ctx->stream));
  double ms = 0; uint32_t n = 0;
  for (size_t i = 0; i + 1 < ctx->ev_used; i += 2) {
    float t = 0;
    QSL_HIP(hipEventElapsedTime(&t, ctx->ev[i], ctx->ev[i + 1]));
    ms += t; ++n;
  }
  ctx->ev_used = 0;
  *total_ms = ms; *launches = n;
  return QSL_OK;
}
