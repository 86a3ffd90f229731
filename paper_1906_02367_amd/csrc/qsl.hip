// qsl.hip -- host side and C ABI of the compression hot path of Qsparse-local-SGD for gfx950; the kernels
// are in the headers included below (qsl_stream.h, qsl_lean.h, qsl_select.h, qsl_encode.h, qsl_dense.h, qsl_decode.h).
//
// One synchronisation step of Algorithm 1 (arXiv:1906.02367) for a batch of R workers:
//   k_stream     v = m + Delta (worker line 1), written over the error memory in ONE pass over HBM;
//                each wave streams one chunk of 1024 coordinates and leaves the coordinates whose
//                rank key reaches the unit's guess in the chunk's own slot (written as one full
//                slot-sized store: no read-modify-write in HBM, no atomic to wait for).  In a segmented
//                context a unit of at most 4096 coordinates has a block of this kernel to itself, which
//                also selects and encodes it.
//   the guess    Top_k: carried from the previous call of the context (k_lean_mark derives it from the
//                candidates it sees); on the first call a quantile of a strided sample of |m + Delta|
//                (k_sample, k_sample_scan).  Rand_k: the rank keys are uniform random words, so it is analytic.
//   k_lean_hist, k_lean_mark, k_lean_emit
//                the guessing units: exact selection of the k largest keys among the candidates (Section 2.2:
//                Top_k / Rand_k, ties to the lower coordinate), the exact ||v_S||_2^2 or ||v_S||_1 (proof of
//                Lemma 1; Lemma 3, m = 1), QSGD levels (Definition 1, example 1) or signs (Definition 2), and
//                the error update m <- v - g on the transmitted coordinates (Algorithm 1, worker line 2)
//   k_lean_one   the same three steps in one launch for a guessing unit that needs only one block
//   k_block_units  a unit too dense for guessing, of at most 40,960 coordinates: all of the above by one block,
//                on a second stream beside the guessing units' kernels
//   k_full       a unit with k = size: nothing to select, the coordinates are copied in order
//   k_select<l>, k_tile_count, k_tile_write, k_quantize
//                exact radix selection (12 + 12 + 8 bits) over the whole vector, ordered compaction and
//                encoding: dense k on a large unit, and the units whose guess failed while the host expects
//                failures (always exact; only the speed depends on the guess)
//   k_pack, k_pack_sent       the packed message (k_pack_sent: QSGD, whose entries of level 0 drop out)
//   k_dense_norm, k_dense_sum, k_dense_scales, k_dense_encode    an operator that keeps every coordinate, with messages that
//                carry no indices: two streaming passes
//   k_aggregate, k_aggregate_entries, k_aggregate_ranges, k_aggregate_dense
//                master line of Algorithm 1, atomic-free, messages added in list order: by look-ups in the other
//                messages (few messages), by coordinate ranges (many), or coordinate by coordinate (every
//                message lists every coordinate)
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
#include <mutex>
#include <new>
#include <vector>

#include "qsl.h"
#include "qsl_device.h"
#include "qsl_layout.h"
#include "qsl_select.h"
#include "qsl_encode.h"
#include "qsl_stream.h"
#include "qsl_lean.h"
#include "qsl_dense.h"
#include "qsl_decode.h"

namespace {
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
  uint32_t nfull_blocks;      // blocks of k_full (per worker): segments with k = size
  uint32_t nnz_hint;          // entries a message is expected to hold at most (sizes the aggregation grid)
  uint32_t* agg_dir;          // [64][agg_ndir] directories of the listed messages (only if messages are expected to be long)
  uint32_t agg_ndir;
  uint32_t n_sampled;         // segments whose guess comes from k_sample
  uint32_t nbig_general;                // how many entries of DevCtx::big_segs are units of the multi-pass kernels (they come first)
  uint32_t nsel_general, ncb_general;   // blocks of the multi-pass kernels without / with (DevCtx::NSEL, NCB) the guessing units' share
  uint32_t n_other;           // segments that k_quantize encodes (not the guessing ones)
  uint32_t warm_R;            // workers whose guessing units carry a guess from an earlier call
  uint32_t safe_left;         // calls still to be made with the multi-pass kernels standing by for failed guesses
  uint32_t* blk_cnt2[2];      // the two arrays of per-block counters of transmitted entries, used in turn
  uint64_t calls;             // compress calls made
  uint32_t nsamp_blocks;      // blocks of the sampling kernel (per worker)
  size_t capacity;
  uint32_t* h_status;         // pinned
  uint32_t* d_nnz_tmp;
  float* own_v;               // [Rmax, d] home of v for calls with m_out = NULL (QSL_FLAG_OWN_V), else null
  hipEvent_t order_ev;        // orders the work of this context across a change of stream
  hipStream_t side;           // the one-block units' kernel runs here, beside the guessing units' kernels
  hipStream_t side2;          // ... and k_lean_one here, when the guessing units with several blocks have kernels of their own
  hipEvent_t join2_ev;
  hipEvent_t fork_ev, join_ev;
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
  if (cfg->sparsifier > 1 || cfg->quantizer > QSL_SIGN_L4) return QSL_ERR_INVALID_ARG;
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
  if ((cfg->flags & QSL_FLAG_DENSE_FORMAT) && K64 != d) return QSL_ERR_INVALID_ARG;      // every segment must keep everything
  *K_out = K64;
  return QSL_OK;
}

// Field widths and sizes of the wire format of an operator (the header of qsl.h describes the format).
struct WireDims {
  uint32_t s, w_idx, w_lev, w_val;
  uint64_t capacity;        // bytes of one message buffer
  uint32_t nnz_hint;        // entries a message is expected to hold at most
};
static WireDims wire_dims(const qsl_config* cfg, uint64_t K) {
  WireDims w;
  const uint32_t L = cfg->num_segments;
  w.s = is_qsgd(cfg->quantizer) ? cfg->s : 1;
  // QSGD drops the entries it rounds to level 0: a segment keeps sum_i min(1, s |v_i| / ||v||_2) <= s sqrt(k)
  // of its k entries on average (Definition 1, example 1, with Cauchy-Schwarz); the other quantisers send all k
  double hint = 0;
  for (uint32_t l = 0; l < L; ++l) {
    const double kl = cfg->seg_k[l];
    hint += is_qsgd(cfg->quantizer) ? std::min(kl, 1.25 * w.s * std::sqrt(kl)) : kl;
  }
  w.nnz_hint = static_cast<uint32_t>(std::min<double>(hint, static_cast<double>(K)));
  const bool dense = (cfg->flags & QSL_FLAG_DENSE_FORMAT) != 0;
  w.w_idx = dense ? 0 : std::max(1u, bit_width_u64(cfg->d - 1));
  // with indices a level 1..s is written as level - 1; without, 0..s as it is
  w.w_lev = is_qsgd(cfg->quantizer) ? bit_width_u64(static_cast<uint64_t>(w.s) - (dense ? 0 : 1)) : 0;
  w.w_val = cfg->quantizer == QSL_FP32 ? 32 : w.w_lev + 1;
  if (dense) w.nnz_hint = static_cast<uint32_t>(K);
  const bool counts = is_qsgd(cfg->quantizer) && L > 1 && !dense;
  uint64_t bits = 32 + 32ull * L + (counts ? 32ull * L : 0);
  bits += align_up(K * w.w_idx, 32) + align_up(K * w.w_val, 32);
  w.capacity = align_up(bits, 64) / 8;
  return w;
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

// Which way a segment goes through the selection, decided from (size, k, sparsifier, flags) alone; fills the fields of
// the plan that follow from that decision (sample layout, static guess, room for candidates) and returns the expected
// number of candidates of a guessing unit (0 otherwise).  sg.size, sg.k and sg.nwt are set by the caller.
static double plan_segment(const qsl_config* cfg, SegInfo& sg) {
  // at most 4096 coordinates: one block; k = size: nothing to select (unless the caller asks for the multi-pass kernels only)
  sg.mode = (sg.nwt <= SMALL_CHUNKS && !(cfg->flags & QSL_FLAG_NO_SMALL_PATH)) ? PATH_SMALL : PATH_GENERAL;
  if (sg.mode != PATH_SMALL && sg.k == sg.size && !(cfg->flags & QSL_FLAG_NO_FAST_PATH)) sg.mode = PATH_FULL;
  sg.T_static = 0xFFFFFFFFu;
  sg.lpc = 8;
  const double n = static_cast<double>(sg.size), p = static_cast<double>(sg.k) / n;
  double cand = 0, slack = 0;                     // expected number of candidates, room beyond 4x that
  if (!(cfg->flags & QSL_FLAG_NO_FAST_PATH) && sg.nwt > SMALL_CHUNKS && sg.mode != PATH_FULL) {
    if (cfg->sparsifier == QSL_TOPK && static_cast<uint64_t>(sg.k) * 64 <= sg.size) {
      // candidates ~ alpha k; the sample must hold enough of them for the guess to sit below the
      // true threshold with ~6.5 sigma: (alpha - 1) sqrt(n_s p) >= 6.5 sqrt(alpha)
      // (a small unit has a small k, so a generous alpha costs few candidates and saves most of the sample)
      // The candidates of a chunk must fit its slot (at most 63, with 4 sigma to spare): a chunk with more sends all
      // of them through the overflow pool, which the selection kernels read entry by entry -- a unit where most
      // chunks do that (k = 1000 of 65,536 with alpha = 3: 47 per chunk) is far slower than on the multi-pass path.
      auto fits = [&](double alpha) { const double pc = alpha * sg.k / sg.nwt; return pc + 4.0 * std::sqrt(pc) <= 63.0; };
      const double alphas[10] = {1.5, 2.0, 3.0, 4.0, 6.0, 8.0, 12.0, 16.0, 24.0, 32.0};
      for (double frac : {1.0 / 16, 1.0 / 4}) {
        for (double alpha : alphas) {
          const double n_s = 42.25 * alpha / ((alpha - 1) * (alpha - 1) * p);
          if (n_s > n * frac || !fits(alpha)) continue;
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
      if (cand == 0 && fits(2.0)) {
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
      if (cand != 0) {                            // else: too dense for the slots, the unit takes the multi-pass kernels
        // Later calls take their guess from the previous call's candidates: the key at rank alpha_w k, far enough below
        // rank k for the count above it to stay above k from one call to the next (6.5 sigma of its own noise, and at
        // least a half more than k for drift).
        double alpha_w = cand / sg.k;
        for (double alpha : alphas)
          if ((alpha - 1) * std::sqrt(static_cast<double>(sg.k)) >= 6.5 * std::sqrt(alpha) && fits(alpha)) { alpha_w = alpha; break; }
        sg.r_warm = static_cast<uint32_t>(std::min<double>(n, std::ceil(alpha_w * sg.k)));
        // where the threshold itself should show in the sample (half the expected count: rather too high than too low)
        sg.r_tau = sg.samp_stride == 64 ? std::max(1u, sg.k / 4)
                                        : std::max(1u, static_cast<uint32_t>(0.5 * sg.n_runs * 64.0 * p));
        sg.r_tau = std::min(sg.r_tau, sg.r_s);
        cand = std::max(cand, alpha_w * sg.k);
        // room for sixteen times the expected candidates: a guess carried over from the last call may lie well below
        // this call's threshold while the error memory is still building up
        sg.d0_cap = static_cast<uint32_t>(std::min<double>(n, 16.0 * cand + slack));
        sg.mode = PATH_FAST;
      }
    } else if (cfg->sparsifier == QSL_RANDK && static_cast<uint64_t>(sg.k) * 16 <= sg.size) {
      // the keys are uniform 32-bit words: keep those above the (1 - q) quantile, q = p + 7 sigma
      const double q = p + 7.0 * std::sqrt(p * (1 - p) / n);
      if (q * CHUNK + 4.0 * std::sqrt(q * CHUNK) <= 63.0) {   // the candidates of a chunk fit its slot with 4 sigma to spare
        sg.T_static = static_cast<uint32_t>(std::floor(4294967296.0 * (1.0 - q)));
        cand = q * n;
        sg.d0_cap = static_cast<uint32_t>(std::min<double>(n, cand + 8.0 * std::sqrt(cand) + 1024.0));
        sg.r_warm = sg.k; sg.r_tau = 1;
        sg.mode = PATH_FAST;
      }
    }
  }
  if (cfg->flags & QSL_FLAG_DENSE_FORMAT) { sg.mode = PATH_FULL; return 0; }   // nothing to select anywhere: two streaming passes
  // too dense to guess, small enough for one block to hold in registers
  if (sg.mode == PATH_GENERAL && sg.size <= BLOCK_MAX && !(cfg->flags & QSL_FLAG_NO_SMALL_PATH)) sg.mode = PATH_SMALL;
  return cand;
}

extern "C" qsl_status qsl_plan_paths(const qsl_config* cfg, uint32_t* path_out) {
  uint64_t K = 0;
  if (!path_out) return QSL_ERR_INVALID_ARG;
  const qsl_status st = check_config(cfg, &K);
  if (st != QSL_OK) return st;
  for (uint32_t l = 0; l < cfg->num_segments; ++l) {
    SegInfo sg;
    memset(&sg, 0, sizeof sg);
    sg.size = cfg->seg_offset[l + 1] - cfg->seg_offset[l];
    sg.k = cfg->seg_k[l];
    sg.nwt = static_cast<uint32_t>((sg.size + CHUNK - 1) / CHUNK);
    (void)plan_segment(cfg, sg);
    path_out[l] = sg.mode;
  }
  return QSL_OK;
}

// releases everything a (possibly half-built) context holds
static void free_ctx(qsl_ctx* ctx) {
  if (ctx->side) { (void)hipStreamSynchronize(ctx->side); (void)hipStreamDestroy(ctx->side); }
  if (ctx->side2) { (void)hipStreamSynchronize(ctx->side2); (void)hipStreamDestroy(ctx->side2); }
  if (ctx->join2_ev) (void)hipEventDestroy(ctx->join2_ev);
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  if (ctx->order_ev) (void)hipEventDestroy(ctx->order_ev);
  if (ctx->fork_ev) (void)hipEventDestroy(ctx->fork_ev);
  if (ctx->join_ev) (void)hipEventDestroy(ctx->join_ev);
  if (ctx->slab) (void)hipFree(ctx->slab);
  if (ctx->h_status) (void)hipHostFree(ctx->h_status);
  delete ctx;
}

extern "C" qsl_status qsl_create(qsl_ctx** out, const qsl_config* cfg, void* hip_stream) {
  uint64_t K64 = 0;
  if (!out) return QSL_ERR_INVALID_ARG;
  const qsl_status cfg_status = check_config(cfg, &K64);
  if (cfg_status != QSL_OK) return cfg_status;
  if (cfg->max_workers == 0 || cfg->max_workers > 1024) return QSL_ERR_INVALID_ARG;
  if (cfg->flags & ~static_cast<uint32_t>(QSL_FLAG_NO_FAST_PATH | QSL_FLAG_NO_SMALL_PATH | QSL_FLAG_OWN_V | QSL_FLAG_NO_WARM_START | QSL_FLAG_DENSE_FORMAT)) return QSL_ERR_INVALID_ARG;
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
  ctx->last_R = 0; ctx->warm_R = 0; ctx->safe_left = 0;
  ctx->timing = 0; ctx->ev_used = 0;
  ctx->slab = nullptr; ctx->h_status = nullptr; ctx->own_v = nullptr; ctx->order_ev = nullptr; ctx->side = nullptr; ctx->side2 = nullptr; ctx->join2_ev = nullptr; ctx->fork_ev = nullptr; ctx->join_ev = nullptr;

  const uint32_t K = static_cast<uint32_t>(K64);
  const WireDims wd = wire_dims(cfg, K64);
  const uint32_t s = wd.s, w_idx = wd.w_idx, w_lev = wd.w_lev, w_val = wd.w_val;
  ctx->nnz_hint = wd.nnz_hint;
  ctx->capacity = static_cast<size_t>(wd.capacity);
  // the kernels count the words of a message in 32 bits
  if (ctx->capacity / 4 > 0xFFFFFFFFull) { delete ctx; return QSL_ERR_UNSUPPORTED; }

  // per-segment plan: single-pass guessing ("fast") where the unit is large and sparse enough
  std::vector<SegInfo>& segs = ctx->segs;
  segs.resize(L);
  std::vector<WtInfo> wts, wts_own;
  std::vector<SelInfo> sels, samps, fulls;
  std::vector<CbInfo> cbs;
  std::vector<uint32_t> fast, smalls;
  uint64_t slot_elems = 0, ovf_entries = 0, d0_entries = 0, nwt64 = 0, nwc = 0;
  uint32_t koff = 0, n_in_stream = 0;
  ctx->n_sampled = 0;
  for (uint32_t l = 0; l < L; ++l) {
    SegInfo& sg = segs[l];
    memset(&sg, 0, sizeof sg);
    sg.start = ctx->off[l]; sg.size = ctx->off[l + 1] - ctx->off[l];
    sg.k = ctx->k[l]; sg.koff = koff; koff += sg.k;
    sg.nwt = static_cast<uint32_t>((sg.size + CHUNK - 1) / CHUNK);
    nwt64 += sg.nwt;
    const double cand = plan_segment(cfg, sg);
    if (L > 1) {
      // The chunks in the order k_stream's waves take them, four to a block.  A unit of at most 4096 coordinates that one
      // block is to select gets its block to itself (filled up with waves that have no chunk), and these blocks come
      // first in the grid: they run longest, so they start before the streaming blocks rather than after them.
      const bool own_block = sg.mode == PATH_SMALL && sg.nwt <= SMALL_CHUNKS;
      std::vector<WtInfo>& list = own_block ? wts_own : wts;
      for (uint32_t t = 0; t < sg.nwt; ++t) {
        WtInfo wi; wi.seg = l; wi.chunk = t; wi.inblock = own_block;
        wi.first = static_cast<uint32_t>(sg.start + static_cast<uint64_t>(t) * CHUNK);
        wi.valid = static_cast<uint16_t>(std::min<uint64_t>(CHUNK, sg.size - static_cast<uint64_t>(t) * CHUNK));
        list.push_back(wi);
      }
      if (own_block) {
        while (wts_own.size() % 4) {
          WtInfo wi; wi.seg = l; wi.chunk = NO_CHUNK; wi.inblock = 1;
          wi.first = static_cast<uint32_t>(sg.start + sg.size); wi.valid = 0;
          wts_own.push_back(wi);
        }
        sg.mode = PATH_SMALL; sg.in_stream = 1;
      }
    }
    if (sg.mode == PATH_FAST && cfg->sparsifier == QSL_TOPK) {        // a guessing Top_k unit samples
      ++ctx->n_sampled;
      for (uint32_t j = 0; j < sg.nsamp; ++j) { SelInfo si; si.seg = l; si.j = j; si.pad0 = si.pad1 = 0; samps.push_back(si); }
    }
    if (sg.mode == PATH_FAST) {
      // the slot of a chunk (64 to 512 bytes) holds the expected candidates with ~4 sigma to spare;
      // chunks that hold more (chance, or clustered large values) spill to an overflow pool that can
      // take every candidate
      // (sized for the calls that take their guess from the call before, i.e. all but the first: r_warm candidates;
      // the sampled guess of a first call may bring up to twice as many, and more of its chunks spill)
      const double steady = cfg->sparsifier == QSL_TOPK ? static_cast<double>(sg.r_warm) : cand;
      const double per_chunk = steady / sg.nwt, need = per_chunk + 4.0 * std::sqrt(per_chunk);
      sg.lpc = need <= 7.0 ? 4 : need <= 15.0 ? 8 : need <= 31.0 ? 16 : 32;
      sg.fidx = static_cast<uint32_t>(fast.size());
      fast.push_back(l);
      sg.slot_off = slot_elems; slot_elems += static_cast<uint64_t>(sg.nwt) * sg.lpc * 2;
      sg.ovf_cap = sg.d0_cap;
      sg.ovf_off = ovf_entries; ovf_entries += sg.ovf_cap;
      sg.d0_off = d0_entries; d0_entries += sg.d0_cap;
      sg.ncb = std::min<uint32_t>(256, (sg.nwt + GGROUP - 1) / GGROUP);    // for the call in which its guess fails
    } else if (sg.mode == PATH_SMALL) {
      if (!sg.in_stream) smalls.push_back(l);       // else a block of k_stream does it
      else ++n_in_stream;
      sg.nsel = 0; sg.ncb = 0;
    } else if (sg.mode == PATH_FULL) {
      const uint64_t ntiles = (sg.size + 4095) / 4096;
      const uint32_t nb = static_cast<uint32_t>(std::min<uint64_t>(ntiles, MAX_FULL_BLOCKS));
      for (uint32_t j = 0; j < nb; ++j) { SelInfo si; si.seg = l; si.j = j; si.pad0 = si.pad1 = 0; fulls.push_back(si); }
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
  // Every unit gets one block; the blocks that are left of the budget go, one at a time, to the unit whose blocks
  // have the most rows to read (the slowest block is the kernel's time).
  {
    auto rows_of = [&](uint32_t l) { return (static_cast<uint64_t>(segs[l].nwt) * segs[l].lpc + 63) / 64; };
    auto want_of = [&](uint32_t l) { return static_cast<uint32_t>(std::min<uint64_t>(MAX_SELECT_BLOCKS, std::max<uint64_t>(1, (rows_of(l) + 47) / 48))); };
    uint64_t used = 0;
    for (uint32_t l : fast) { segs[l].nsel = 1; used += ctx->Rmax; }
    auto load = [&](uint32_t l) { return static_cast<double>(rows_of(l)) / segs[l].nsel; };
    auto lighter = [&](uint32_t a, uint32_t b) { return load(a) < load(b); };
    std::vector<uint32_t> heap;
    for (uint32_t l : fast) if (want_of(l) > 1) heap.push_back(l);
    std::make_heap(heap.begin(), heap.end(), lighter);
    const uint64_t budget = 256;                     // measured: 384, 512 and 768 are no faster on segmented contexts and slower on one segment
    while (!heap.empty() && used + ctx->Rmax <= budget) {
      std::pop_heap(heap.begin(), heap.end(), lighter);
      const uint32_t l = heap.back();
      ++segs[l].nsel; used += ctx->Rmax;
      if (segs[l].nsel < want_of(l)) std::push_heap(heap.begin(), heap.end(), lighter); else heap.pop_back();
    }
  }
  // The block lists of the multi-pass kernels: the units that always take them first, then the guessing units, whose
  // share is launched only while the host expects failed guesses.  A guessing unit's blocks are also the blocks of
  // k_lean_* (fsels).
  std::vector<SelInfo> fsels, sels_f;
  // A guessing unit with a single block takes k_lean_one: one launch instead of three.
  const bool one_kernel = true;
  std::vector<CbInfo> cbs_f;
  uint32_t cb_slots = 0;
  for (uint32_t l = 0; l < L; ++l) {
    SegInfo& sg = segs[l];
    const bool guessing = sg.mode == PATH_FAST;
    for (uint32_t j = 0; j < sg.nsel; ++j) {
      SelInfo si; si.seg = l; si.j = j; si.pad0 = si.pad1 = 0;
      (guessing ? sels_f : sels).push_back(si);
      if (guessing && (sg.nsel > 1 || !one_kernel)) fsels.push_back(si);      // (else the unit goes to k_lean_one)
    }
    sg.wc_base = static_cast<uint32_t>(nwc); nwc += sg.nsel * (BIG / 64);
    sg.cb_base = cb_slots; cb_slots += sg.ncb;
    for (uint32_t b = 0; b < sg.ncb; ++b) { CbInfo ci; ci.seg = l; ci.b = b; ci.pad0 = ci.pad1 = 0; (guessing ? cbs_f : cbs).push_back(ci); }
  }
  // The launch lists in decreasing order of a block's work: the blocks of a kernel start over several microseconds
  // (the waves of a few hundred 1024-thread blocks), and the kernel ends when the slowest block does, so the heavy
  // blocks go first.  A multi-pass block weighs its chunks (every coordinate meets an LDS atomic), a guessing block
  // its slot rows, a compaction block of the dense list one tile.
  auto select_cost = [&](const SelInfo& si) {
    const SegInfo& sg = segs[si.seg];
    if (sg.mode == PATH_FAST) return 1.2 * static_cast<double>((static_cast<uint64_t>(sg.nwt) * sg.lpc + 63) / 64) / sg.nsel / 16.0;
    return 0.8 * static_cast<double>(sg.nwt) / sg.nsel;
  };
  auto by_select_cost = [&](const SelInfo& a, const SelInfo& b) { return select_cost(a) > select_cost(b); };
  std::stable_sort(sels.begin(), sels.end(), by_select_cost);
  std::stable_sort(fsels.begin(), fsels.end(), by_select_cost);
  std::vector<uint32_t> ones;                       // guessing segments whose units have a single block, heaviest first
  for (uint32_t l : fast) if (segs[l].nsel == 1 && one_kernel) ones.push_back(l);
  std::stable_sort(ones.begin(), ones.end(), [&](uint32_t a, uint32_t b) {
    return static_cast<uint64_t>(segs[a].nwt) * segs[a].lpc > static_cast<uint64_t>(segs[b].nwt) * segs[b].lpc; });
  auto general_cost = [&](uint32_t seg) { return static_cast<double>(segs[seg].nwt) / segs[seg].nsel; };
  std::stable_sort(sels_f.begin(), sels_f.end(), [&](const SelInfo& a, const SelInfo& b) { return general_cost(a.seg) > general_cost(b.seg); });
  auto compact_cost = [&](const CbInfo& ci) {
    const SegInfo& sg = segs[ci.seg];
    return std::max(1.0, static_cast<double>((sg.nwt + GGROUP - 1) / GGROUP) / sg.ncb);
  };
  auto by_compact_cost = [&](const CbInfo& a, const CbInfo& b) { return compact_cost(a) > compact_cost(b); };
  std::stable_sort(cbs.begin(), cbs.end(), by_compact_cost);
  std::stable_sort(cbs_f.begin(), cbs_f.end(), by_compact_cost);
  ctx->nsel_general = static_cast<uint32_t>(sels.size());
  ctx->ncb_general = static_cast<uint32_t>(cbs.size());
  sels.insert(sels.end(), sels_f.begin(), sels_f.end());
  cbs.insert(cbs.end(), cbs_f.begin(), cbs_f.end());
  ctx->n_other = L - static_cast<uint32_t>(fast.size()) - static_cast<uint32_t>(smalls.size()) - n_in_stream;   // what k_quantize encodes
  // a sample block's work: its share of the unit's runs (or chunks, when the whole unit is read); a small unit's: its size
  auto sample_cost = [&](const SelInfo& si) {
    const SegInfo& sg = segs[si.seg];
    return (sg.samp_stride == 64 ? 16.0 * sg.nwt : static_cast<double>(sg.n_runs)) / sg.nsamp;
  };
  std::stable_sort(samps.begin(), samps.end(), [&](const SelInfo& a, const SelInfo& b) { return sample_cost(a) > sample_cost(b); });
  std::stable_sort(smalls.begin(), smalls.end(), [&](uint32_t a, uint32_t b) { return segs[a].size > segs[b].size; });
  ctx->nsamp_blocks = static_cast<uint32_t>(samps.size());
  if (L > 1) {                                      // the small units' own blocks first, with their fillers
    wts.insert(wts.begin(), wts_own.begin(), wts_own.end());
    nwt64 = wts.size();
  }
  const uint32_t NWT = static_cast<uint32_t>(nwt64);
  const uint32_t NSEL = static_cast<uint32_t>(sels.size()), NCB = static_cast<uint32_t>(cbs.size());
  const uint32_t NSELF = static_cast<uint32_t>(fsels.size());
  const uint32_t NWC = static_cast<uint32_t>(nwc);
  const uint32_t QB = (K + BLOCK - 1) / BLOCK;
  const uint64_t R = ctx->Rmax, U = R * L;

  // one slab, carved; the part that must be zero between calls comes first
  uint64_t bytes = 0;
  auto carve = [&](uint64_t n) { const uint64_t o = bytes; bytes = align_up(bytes + n, 256); return o; };
  const uint64_t o_hist = carve(4ull * 3 * HBINS * U), o_ctr = carve(4ull * CTR_LINES * PAD * U);
  const uint64_t o_acc = carve(8ull * ACC_SLOTS * U), o_status = carve(8);
  const uint64_t o_blk = carve(4ull * QB * R * 2);    // the two arrays of per-block counters of transmitted entries
  const uint64_t zero_bytes = bytes;
  const uint64_t o_segs = carve(sizeof(SegInfo) * L), o_wts = carve(sizeof(WtInfo) * std::max<size_t>(1, wts.size()));
  const uint64_t o_sels = carve(sizeof(SelInfo) * NSEL), o_cbs = carve(sizeof(CbInfo) * NCB);
  const uint64_t o_samps = carve(sizeof(SelInfo) * samps.size());
  const uint64_t o_fsels = carve(sizeof(SelInfo) * std::max<size_t>(1, fsels.size()));
  const uint64_t o_ones = carve(4ull * std::max<size_t>(1, ones.size()));
  const uint64_t o_fulls = carve(sizeof(SelInfo) * std::max<size_t>(1, fulls.size()));
  const uint64_t o_fast = carve(4ull * std::max<size_t>(1, fast.size()));
  const uint64_t o_small = carve(4ull * std::max<size_t>(1, smalls.size()));
  std::vector<uint32_t> bigs;
  // the units that use the three histograms in memory: those of the multi-pass kernels first, then the guessing ones
  // (whose only histogram k_lean_emit clears itself, unless the multi-pass kernels stood by for them in that call)
  for (uint32_t l = 0; l < L; ++l) if (segs[l].mode == PATH_GENERAL) bigs.push_back(l);
  ctx->nbig_general = static_cast<uint32_t>(bigs.size());
  for (uint32_t l = 0; l < L; ++l) if (segs[l].mode == PATH_FAST) bigs.push_back(l);
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
  std::vector<uint32_t> seg_start(L), seg_koff(L), seg_whole(L);
  for (uint32_t l = 0; l < L; ++l) { seg_start[l] = static_cast<uint32_t>(segs[l].start); seg_koff[l] = segs[l].koff; seg_whole[l] = segs[l].k == segs[l].size; }
  const uint64_t o_sstart = carve(4ull * L), o_skoff = carve(4ull * L), o_swhole = carve(4ull * L);
  const uint64_t o_units = carve(sizeof(UnitState) * U);
  const uint64_t o_slots = carve(8ull * std::max<uint64_t>(2, slot_elems) * R);
  const uint64_t o_ovf = carve(8ull * std::max<uint64_t>(1, ovf_entries) * R);
  const bool randk = cfg->sparsifier == QSL_RANDK;
  const uint64_t o_skey = carve(randk ? 4ull * std::max<uint64_t>(2, slot_elems) * R : 4);
  const uint64_t o_okey = carve(randk ? 4ull * std::max<uint64_t>(1, ovf_entries) * R : 4);
  const uint64_t o_d0 = carve(8ull * std::max<uint64_t>(1, d0_entries) * R);
  const uint64_t o_d0k = carve(4ull * std::max<uint64_t>(1, d0_entries) * R);
  const uint64_t o_wc = carve(4ull * NWC * R), o_ws = carve(4ull * NWC * R), o_cbc = carve(8ull * NCB * R);
  const uint64_t o_tlist = carve(16ull * LISTCAP * std::max<size_t>(1, fast.size()) * R);
  const bool dense = (cfg->flags & QSL_FLAG_DENSE_FORMAT) != 0;
  const uint64_t KA = dense ? 1 : K;                 // the index-free format needs no per-entry arrays
  const uint64_t o_si = carve(4ull * KA * R), o_sv = carve(4ull * KA * R), o_sc = carve(4ull * KA * R);
  const uint64_t o_pre = carve(4ull * (QB + 1) * R);
  const uint64_t KV = is_qsgd(cfg->quantizer) ? 1 : KA;     // the final arrays of the quantisers that send every selected coordinate
  const uint64_t o_vi = carve(4ull * KV * R), o_vc = carve(4ull * KV * R);
  const uint64_t o_tmp = carve(4ull * 1024);
  ctx->agg_ndir = static_cast<uint32_t>(((d + (1u << AGG_DIR_SHIFT) - 1) >> AGG_DIR_SHIFT) + 1);
  const bool want_dir = true;                       // (6.4 MB for 25.6 M coordinates)
  const uint64_t o_dir = carve(4ull * 65 * ctx->agg_ndir);       // 64 directories and the list of crowded ranges
  const uint64_t o_ownv = carve((cfg->flags & QSL_FLAG_OWN_V) ? 4ull * R * d : 4);
  const uint64_t dense_nb = dense ? std::min<uint64_t>((d + DTILE - 1) / DTILE, MAX_DENSE_BLOCKS) : 0;
  const uint64_t o_dpart = carve(8ull * R * ACC_SLOTS * dense_nb + 8), o_dtag = carve(4ull * R * dense_nb + 4);
  if (hipMalloc(&ctx->slab, bytes) != hipSuccess) { ctx->slab = nullptr; free_ctx(ctx); return QSL_ERR_DEVICE; }
  char* base = static_cast<char*>(ctx->slab);
  bool ok = hipMemset(base, 0, zero_bytes) == hipSuccess;
  auto upload = [&](uint64_t o, const void* src, size_t n) {
    if (n) ok = ok && hipMemcpy(base + o, src, n, hipMemcpyHostToDevice) == hipSuccess;
  };
  upload(o_segs, segs.data(), sizeof(SegInfo) * L);
  upload(o_wts, wts.data(), sizeof(WtInfo) * wts.size());
  upload(o_sels, sels.data(), sizeof(SelInfo) * NSEL);
  upload(o_samps, samps.data(), sizeof(SelInfo) * samps.size());
  upload(o_fsels, fsels.data(), sizeof(SelInfo) * fsels.size());
  upload(o_ones, ones.data(), 4ull * ones.size());
  upload(o_fulls, fulls.data(), sizeof(SelInfo) * fulls.size());
  upload(o_cbs, cbs.data(), sizeof(CbInfo) * NCB);
  upload(o_fast, fast.data(), 4 * fast.size());
  upload(o_small, smalls.data(), 4 * smalls.size());
  upload(o_big, bigs.data(), 4 * bigs.size());
  upload(o_segdir, seg_dir.data(), 4 * seg_dir.size());
  upload(o_slotdir, slot_dir.data(), 4 * slot_dir.size());
  upload(o_sstart, seg_start.data(), 4ull * L);
  upload(o_skoff, seg_koff.data(), 4ull * L);
  upload(o_swhole, seg_whole.data(), 4ull * L);
  ok = ok && hipHostMalloc(reinterpret_cast<void**>(&ctx->h_status), 64, hipHostMallocMapped) == hipSuccess;
  // The events order work on one device (what a kernel wrote is visible device-wide when it ends), so they need no
  // system-scope fence when they complete: with one, every record costs the stream 2-3 us (measured: a round with the
  // two timing events 442 -> 437 us, the 161-tensor round with fork and join 548 -> 542 us).
  const unsigned evf = hipEventDisableTiming | hipEventDisableSystemFence;
  ok = ok && hipEventCreateWithFlags(&ctx->order_ev, evf) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&ctx->fork_ev, evf) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&ctx->join_ev, evf) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&ctx->join2_ev, evf) == hipSuccess;
  ok = ok && hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) == hipSuccess;      // default priority
  ok = ok && hipStreamCreateWithFlags(&ctx->side2, hipStreamNonBlocking) == hipSuccess;
  ok = ok && hipDeviceSynchronize() == hipSuccess;
  if (!ok) { free_ctx(ctx); return QSL_ERR_DEVICE; }

  DevCtx& c = ctx->dc;
  c.segs = reinterpret_cast<const SegInfo*>(base + o_segs);
  c.wts = reinterpret_cast<const WtInfo*>(base + o_wts);
  c.sels = reinterpret_cast<const SelInfo*>(base + o_sels);
  c.samps = reinterpret_cast<const SelInfo*>(base + o_samps);
  c.fsels = reinterpret_cast<const SelInfo*>(base + o_fsels);
  c.one_segs = reinterpret_cast<const uint32_t*>(base + o_ones); c.none = static_cast<uint32_t>(ones.size());
  c.cbs = reinterpret_cast<const CbInfo*>(base + o_cbs);
  c.fast_segs = reinterpret_cast<const uint32_t*>(base + o_fast);
  c.small_segs = reinterpret_cast<const uint32_t*>(base + o_small);
  c.big_segs = reinterpret_cast<const uint32_t*>(base + o_big); c.nbig = static_cast<uint32_t>(bigs.size());
  c.seg_dir = reinterpret_cast<const uint32_t*>(base + o_segdir);
  c.slot_dir = reinterpret_cast<const uint32_t*>(base + o_slotdir);
  c.seg_start = reinterpret_cast<const uint32_t*>(base + o_sstart); c.seg_koff = reinterpret_cast<const uint32_t*>(base + o_skoff);
  c.seg_whole = reinterpret_cast<const uint32_t*>(base + o_swhole);
  ctx->nsmall = static_cast<uint32_t>(smalls.size()); c.nblock = ctx->nsmall;
  c.fulls = reinterpret_cast<const SelInfo*>(base + o_fulls);
  ctx->nfull_blocks = static_cast<uint32_t>(fulls.size());
  c.units = reinterpret_cast<UnitState*>(base + o_units);
  c.slots = reinterpret_cast<uint2*>(base + o_slots); c.slot_stride = std::max<uint64_t>(2, slot_elems);
  c.ovf = reinterpret_cast<uint2*>(base + o_ovf); c.ovf_stride = std::max<uint64_t>(1, ovf_entries);
  c.slot_key = reinterpret_cast<uint32_t*>(base + o_skey); c.ovf_key = reinterpret_cast<uint32_t*>(base + o_okey);
  c.d0 = reinterpret_cast<uint2*>(base + o_d0); c.d0_key = reinterpret_cast<uint32_t*>(base + o_d0k);
  c.d0_stride = std::max<uint64_t>(1, d0_entries);
  c.wave_cnt = reinterpret_cast<uint32_t*>(base + o_wc); c.wave_sel = reinterpret_cast<uint32_t*>(base + o_ws);
  c.cb_cnt = reinterpret_cast<uint2*>(base + o_cbc);
  c.tlist = reinterpret_cast<uint4*>(base + o_tlist);
  ctx->h_status[8] = 0;
  {
    void* dflag = nullptr;                          // the device's address of a word of the pinned host block
    if (hipHostGetDevicePointer(&dflag, ctx->h_status + 8, 0) != hipSuccess || !dflag) { free_ctx(ctx); return QSL_ERR_DEVICE; }
    c.host_flag = static_cast<uint32_t*>(dflag);
  }
  c.hist = reinterpret_cast<uint32_t*>(base + o_hist); c.ctr = reinterpret_cast<uint32_t*>(base + o_ctr);
  c.norm_acc = reinterpret_cast<uint64_t*>(base + o_acc);
  c.sel_idx = reinterpret_cast<uint32_t*>(base + o_si); c.sel_val = reinterpret_cast<uint32_t*>(base + o_sv);
  c.sel_code = reinterpret_cast<uint32_t*>(base + o_sc);
  ctx->blk_cnt2[0] = reinterpret_cast<uint32_t*>(base + o_blk); ctx->blk_cnt2[1] = ctx->blk_cnt2[0] + QB * R;
  ctx->calls = 0;
  c.blk_cnt = ctx->blk_cnt2[0]; c.blk_cnt_next = ctx->blk_cnt2[1]; c.Rmax = ctx->Rmax;
  c.blk_pre = reinterpret_cast<uint32_t*>(base + o_pre);
  c.surv_idx = reinterpret_cast<uint32_t*>(base + o_vi); c.surv_code = reinterpret_cast<uint32_t*>(base + o_vc);
  c.status = reinterpret_cast<uint32_t*>(base + o_status);
  c.dense_part = reinterpret_cast<uint64_t*>(base + o_dpart); c.dense_tag = reinterpret_cast<uint32_t*>(base + o_dtag);
  ctx->d_nnz_tmp = reinterpret_cast<uint32_t*>(base + o_tmp);
  ctx->agg_dir = want_dir ? reinterpret_cast<uint32_t*>(base + o_dir) : nullptr;
  ctx->own_v = (cfg->flags & QSL_FLAG_OWN_V) ? reinterpret_cast<float*>(base + o_ownv) : nullptr;
  c.d = d; c.seed = cfg->seed; c.L = L; c.K = K; c.NWT = NWT; c.NSEL = NSEL; c.NCB = NCB; c.NWC = NWC; c.QB = QB;
  c.NSELF = NSELF; c.nfast = static_cast<uint32_t>(fast.size()); c.s = s; c.w_idx = w_idx; c.w_lev = w_lev; c.w_val = w_val;
  c.sparsifier = cfg->sparsifier; c.quantizer = cfg->quantizer; c.dense = dense;
  c.cap_words = static_cast<uint32_t>(ctx->capacity / 4);
  ctx->one.start = 0; ctx->one.size = segs[0].size; ctx->one.slot_off = 0; ctx->one.ovf_off = 0;
  ctx->one.lpc = segs[0].lpc; ctx->one.ovf_cap = segs[0].ovf_cap;
  k_init<<<dim3(static_cast<uint32_t>((U + 255) / 256)), 256, 0, ctx->stream>>>(c, static_cast<uint32_t>(U));
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) { free_ctx(ctx); return QSL_ERR_DEVICE; }
  *out = ctx;
  return QSL_OK;
}

extern "C" qsl_status qsl_destroy(qsl_ctx* ctx) {
  if (!ctx) return QSL_ERR_INVALID_ARG;
  (void)hipStreamSynchronize(ctx->stream);
  free_ctx(ctx);
  return QSL_OK;
}

extern "C" qsl_status qsl_set_stream(qsl_ctx* ctx, void* hip_stream) {
  if (!ctx) return QSL_ERR_INVALID_ARG;
  hipStream_t next = static_cast<hipStream_t>(hip_stream);
  if (next != ctx->stream) {
    // the calls of a context share its scratch: what is already enqueued on the old stream must finish before
    // anything enqueued on the new one starts
    QSL_HIP(hipEventRecord(ctx->order_ev, ctx->stream));
    QSL_HIP(hipStreamWaitEvent(next, ctx->order_ev, 0));
    ctx->stream = next;
  }
  return QSL_OK;
}

extern "C" size_t qsl_msg_capacity_bytes(const qsl_ctx* ctx) { return ctx ? ctx->capacity : 0; }

// An operator that keeps every coordinate, index-free messages: two streaming passes (qsl_dense.h).
static qsl_status launch_dense(qsl_ctx* ctx, const float* m, const float* delta, const float* xm, float* m_out,
                               uint32_t worker0, uint32_t R, uint64_t round, uint8_t* msg, uint64_t* msg_bits,
                               uint32_t* sel_idx, uint16_t* sel_level) {
  const DevCtx& c = ctx->dc;
  hipStream_t st = ctx->stream;
  const uint64_t ntiles = (c.d + DTILE - 1) / DTILE;
  const dim3 grid(static_cast<uint32_t>(std::min<uint64_t>(ntiles, MAX_DENSE_BLOCKS)), R);
  const bool timed = ctx->timing != 0;
  if (timed) {
    if (ctx->ev_used + 2 > ctx->ev.size()) {
      for (int i = 0; i < 2; ++i) { hipEvent_t e; QSL_HIP(hipEventCreateWithFlags(&e, hipEventDisableSystemFence)); ctx->ev.push_back(e); }
    }
    QSL_HIP(hipEventRecord(ctx->ev[ctx->ev_used], st));
  }
  if (xm == nullptr) k_dense_norm<false><<<grid, BLOCK, 0, st>>>(c, m, delta, xm, m_out);
  else k_dense_norm<true><<<grid, BLOCK, 0, st>>>(c, m, delta, xm, m_out);
  if (timed) { QSL_HIP(hipEventRecord(ctx->ev[ctx->ev_used + 1], st)); ctx->ev_used += 2; }
  if (c.quantizer != QSL_FP32) k_dense_sum<<<dim3((grid.x + SUM_ROWS - 1) / SUM_ROWS, R), SUM_BLOCK, 0, st>>>(c, grid.x);
  const uint32_t U = R * c.L;
  k_dense_scales<<<dim3((U + BLOCK / 64 - 1) / (BLOCK / 64)), BLOCK, 0, st>>>(c, U);
  const dim3 egrid(static_cast<uint32_t>(std::min<uint64_t>(ntiles, MAX_ENCODE_BLOCKS)), R);
  k_dense_encode<<<egrid, BLOCK, 0, st>>>(c, m_out, worker0, round, msg, msg_bits, sel_idx, sel_level);
  QSL_HIP(hipGetLastError());
  return QSL_OK;
}

template <int SPARS>
static qsl_status launch_compress(qsl_ctx* ctx, const float* m, const float* delta, const float* xm, float* m_out,
                                  uint32_t worker0,
                                  uint32_t R, uint64_t round, uint8_t* msg, uint64_t* msg_bits, uint32_t* sel_idx,
                                  uint16_t* sel_level) {
  DevCtx& c = ctx->dc;
  hipStream_t st = ctx->stream;
  if (static_cast<uint64_t>(std::max(std::max(c.NSEL, c.NCB), std::max(std::max(ctx->nsamp_blocks, c.nblock), c.NSELF + c.nfast + c.none))) * R > 0x7FFFFFFFull)
    return QSL_ERR_UNSUPPORTED;                    // the list kernels use one-dimensional grids of (list entries x workers)
  if (xm != nullptr && static_cast<uint64_t>(((c.NWT + 3) / 4 + 7) / 8) * 8 * R > 0x7FFFFFFFull)
    return QSL_ERR_UNSUPPORTED;                    // ... and so does the streaming kernel when it reads x_t
  c.blk_cnt = ctx->blk_cnt2[ctx->calls & 1]; c.blk_cnt_next = ctx->blk_cnt2[(ctx->calls & 1) ^ 1];
  ++ctx->calls;
  // A kernel that had to resolve a failed guess with one block (slow for a large unit) leaves a word in pinned host
  // memory; the next calls then keep the multi-pass kernels standing by for the units whose guess fails.  The word
  // may be seen a few calls late: only speed depends on it, never the result.
  if (ctx->h_status[8] != 0) { ctx->h_status[8] = 0; ctx->safe_left = 16; }
  const bool safe = ctx->safe_left > 0;
  if (safe) --ctx->safe_left;
  const bool cold = ctx->warm_R < R || (ctx->cfg.flags & QSL_FLAG_NO_WARM_START) != 0;
  if (SPARS == QSL_TOPK && ctx->n_sampled > 0 && cold) {
    k_sample<<<dim3(ctx->nsamp_blocks * R), BIG, 0, st>>>(c, m, delta, xm, R);
    k_sample_scan<<<dim3(c.nfast, R), BIG, 0, st>>>(c);
  }
  ctx->warm_R = std::max(ctx->warm_R, R);
  const bool timed = ctx->timing != 0;
  if (timed) {
    if (ctx->ev_used + 2 > ctx->ev.size()) {
      for (int i = 0; i < 2; ++i) { hipEvent_t e; QSL_HIP(hipEventCreateWithFlags(&e, hipEventDisableSystemFence)); ctx->ev.push_back(e); }
    }
    QSL_HIP(hipEventRecord(ctx->ev[ctx->ev_used], st));
  }
  const uint32_t nblk = (c.NWT + 3) / 4;
  // QSGD: k_pack_sent adds the fields of the transmitted entries to messages that the streaming pass has cleared
  uint32_t* msg_zero = is_qsgd(c.quantizer) ? reinterpret_cast<uint32_t*>(msg) : nullptr;
  if (xm == nullptr) {
    const dim3 sgrid(nblk, R);
    if (c.L == 1) k_stream<SPARS, true, false><<<sgrid, BLOCK, 0, st>>>(c, ctx->one, m, delta, xm, m_out, worker0, round, R, msg_zero, sel_idx, sel_level);
    else k_stream<SPARS, false, false><<<sgrid, BLOCK, 0, st>>>(c, ctx->one, m, delta, xm, m_out, worker0, round, R, msg_zero, sel_idx, sel_level);
  } else {
    const dim3 sgrid(static_cast<uint32_t>(static_cast<uint64_t>((nblk + 7) / 8) * 8 * R));     // checked above
    if (c.L == 1) k_stream<SPARS, true, true><<<sgrid, BLOCK, 0, st>>>(c, ctx->one, m, delta, xm, m_out, worker0, round, R, msg_zero, sel_idx, sel_level);
    else k_stream<SPARS, false, true><<<sgrid, BLOCK, 0, st>>>(c, ctx->one, m, delta, xm, m_out, worker0, round, R, msg_zero, sel_idx, sel_level);
  }
  if (timed) { QSL_HIP(hipEventRecord(ctx->ev[ctx->ev_used + 1], st)); ctx->ev_used += 2; }

  // Units that a single block selects and encodes whole need nothing but v: their kernel runs on a stream of the
  // context's own beside the kernels of the other units (one block works tens of microseconds on a unit of 40,960
  // coordinates) and is joined before the messages are put together.
  // With k_lean_one in the call the roles are swapped: the block units start on the caller's stream at once and
  // k_lean_one follows on the second stream behind the event -- its blocks take a compute unit each (123 registers),
  // so whichever kernel is dispatched first keeps the other waiting, and the block units are the longer (measured on
  // the 161-tensor table: k_lean_one first 541-548 us per round, the three kernels 536 us).  Not while failed guesses
  // are expected: the multi-pass kernels on the caller's stream read what k_lean_one finds out about its units.
  // ... nor when some guessing units have several blocks: their three kernels would wait on the caller's stream behind
  // the block units (161 tensors, one worker: 160 us per round that way, against 133 us with the block units on the second stream).
  const bool swapped = c.nblock != 0 && c.none != 0 && c.NSELF == 0 && !safe;
  const bool forked = c.nblock != 0 && !swapped && (c.NSELF != 0 || c.none != 0 || ctx->n_other != 0);
  // Guessing units of both kinds in one call (a single block: k_lean_one; several: the three kernels) and no block units:
  // k_lean_one goes to a stream of its own, beside the three kernels (160 tensors, one worker: 115 -> 106 us per round,
  // two workers 171 -> 162 us).  Beside k_block_units as well, three kernels at once, it loses (161 tensors, one worker:
  // 127 -> 134 us; four workers 293 -> 302 us).
  const bool one_aside = c.none != 0 && c.NSELF != 0 && c.nblock == 0 && !safe;
  if (swapped) {
    QSL_HIP(hipEventRecord(ctx->fork_ev, st));
    QSL_HIP(hipStreamWaitEvent(ctx->side, ctx->fork_ev, 0));
    k_block_units<SPARS><<<dim3(c.nblock * R), BIG, 0, st>>>(c, R, m_out, worker0, round, sel_idx, sel_level);
    k_lean_one<SPARS><<<dim3(c.none * R), BIG, 0, ctx->side>>>(c, ctx->segs[0], R, m_out, worker0, round, sel_idx, sel_level, 0);
    QSL_HIP(hipEventRecord(ctx->join_ev, ctx->side));
  } else if (c.nblock) {
    hipStream_t bs = st;
    if (forked) {
      QSL_HIP(hipEventRecord(ctx->fork_ev, st));
      QSL_HIP(hipStreamWaitEvent(ctx->side, ctx->fork_ev, 0));
      bs = ctx->side;
    }
    k_block_units<SPARS><<<dim3(c.nblock * R), BIG, 0, bs>>>(c, R, m_out, worker0, round, sel_idx, sel_level);
    if (forked) QSL_HIP(hipEventRecord(ctx->join_ev, ctx->side));
  }
  if (one_aside) {
    if (!forked) QSL_HIP(hipEventRecord(ctx->fork_ev, st));
    QSL_HIP(hipStreamWaitEvent(ctx->side2, ctx->fork_ev, 0));
    k_lean_one<SPARS><<<dim3(c.none * R), BIG, 0, ctx->side2>>>(c, ctx->segs[0], R, m_out, worker0, round, sel_idx, sel_level, 0);
    QSL_HIP(hipEventRecord(ctx->join2_ev, ctx->side2));
  }
  if (ctx->nfull_blocks) k_full<<<dim3(ctx->nfull_blocks, R), BLOCK, 0, st>>>(c, m_out);
  // guessing units of a single block: the whole way from the slots to the encoded entries in one launch
  if (c.none && !swapped && !one_aside) k_lean_one<SPARS><<<dim3(c.none * R), BIG, 0, st>>>(c, ctx->segs[0], R, m_out, worker0, round, sel_idx, sel_level, safe ? 1 : 0);
  if (c.NSELF) {                                   // guessing units: candidates' histogram, threshold bin and dense list
    k_lean_hist<SPARS><<<dim3(c.NSELF * R), BIG, 0, st>>>(c, ctx->segs[0], R);
    k_lean_mark<SPARS><<<dim3(c.NSELF * R), BIG, 0, st>>>(c, ctx->segs[0], R);
  }
  // the multi-pass kernels: a launch per digit and two for the compaction, for the units planned that way -- and for
  // the guessing units too while failed guesses are expected
  const uint32_t nsel = safe ? c.NSEL : ctx->nsel_general, ncb = safe ? c.NCB : ctx->ncb_general;
  if (nsel) {
    k_select<0, SPARS><<<dim3(nsel * R), BIG, 0, st>>>(c, ctx->segs[0], m_out, worker0, round, R);
    k_select<1, SPARS><<<dim3(nsel * R), BIG, 0, st>>>(c, ctx->segs[0], m_out, worker0, round, R);
    k_select<2, SPARS><<<dim3(nsel * R), BIG, 0, st>>>(c, ctx->segs[0], m_out, worker0, round, R);
    k_tile_count<SPARS><<<dim3(ncb * R), BLOCK, 0, st>>>(c, ctx->segs[0], m_out, worker0, round, R);
    k_tile_write<SPARS><<<dim3(ncb * R), BLOCK, 0, st>>>(c, ctx->segs[0], m_out, worker0, round, R);
  }
  if (ctx->n_other || safe) k_quantize<<<dim3(c.QB, R), BLOCK, 0, st>>>(c, m_out, worker0, round, sel_idx, sel_level, safe ? 1 : 0);
  // the guessing units' exact threshold, ordered output and codes; one more block per guessing unit for failures
  if (c.NSELF)
    k_lean_emit<SPARS><<<dim3((c.NSELF + c.nfast) * R), BIG, 0, st>>>(c, ctx->segs[0], R, c.NSELF * R, m_out, worker0, round,
                                                                     sel_idx, sel_level, safe ? 1 : 0);
  if (forked || swapped) QSL_HIP(hipStreamWaitEvent(st, ctx->join_ev, 0));
  if (one_aside) QSL_HIP(hipStreamWaitEvent(st, ctx->join2_ev, 0));
  const uint32_t nzero = safe ? c.nbig : ctx->nbig_general;
  if (is_qsgd(c.quantizer)) {                      // entries may drop out: the message from the selected arrays, a block per 256 slots
    if (c.QB > MAX_QB_INLINE) k_surv_scan<<<dim3(R), 1024, 0, st>>>(c);
    k_pack_sent<<<dim3(c.QB, R), BLOCK, 0, st>>>(c, msg, msg_bits, nzero);
  } else {                                         // every selected coordinate is sent: the final arrays are written already
    // a thread per message word -- two words per thread once the blocks would no longer all be resident at once (2048
    // blocks of 256 threads): a kernel of many short threads is bound by the rate at which its waves start (161 tensors,
    // 99,400 entries, 8 workers: 13.0 us with one word per thread, 10.2 us with two, 11.2 with four, 14.3 with eight; with
    // a quarter of the entries one word per thread is the faster by 1.5 us)
    uint32_t pack_blocks = (c.cap_words + BLOCK - 1) / BLOCK;
    if (static_cast<uint64_t>(pack_blocks) * R > 2048) pack_blocks = (pack_blocks + 1) / 2;
    k_pack<<<dim3(pack_blocks, R), BLOCK, 0, st>>>(c, msg, msg_bits, nzero);
  }
  QSL_HIP(hipGetLastError());
  return QSL_OK;
}

static qsl_status compress_checked(qsl_ctx* ctx, const float* m, const float* delta, const float* xm, float* m_out,
                                   uint32_t worker0, uint32_t R, uint64_t round, uint8_t* msg, uint64_t* msg_bits,
                                   uint32_t* sel_idx, uint16_t* sel_level) {
  if (!ctx || !m || !delta || !msg || R == 0 || R > ctx->Rmax || (round >> 62)) return QSL_ERR_INVALID_ARG;
  if (!m_out) m_out = ctx->own_v;                  // "send g, leave m alone": v lives in the context's own array
  if (!m_out) return QSL_ERR_INVALID_ARG;
  if (static_cast<uint64_t>(worker0) + R > (1ull << 32)) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(delta) | reinterpret_cast<uintptr_t>(m_out) |
       reinterpret_cast<uintptr_t>(xm) | reinterpret_cast<uintptr_t>(sel_idx)) & 3) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(msg) | reinterpret_cast<uintptr_t>(msg_bits)) & 7) return QSL_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(sel_level) & 1) return QSL_ERR_INVALID_ARG;
  ctx->last_R = R;
  if (ctx->dc.dense) return launch_dense(ctx, m, delta, xm, m_out, worker0, R, round, msg, msg_bits, sel_idx, sel_level);
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

// the listed rows, checked: a message may be listed once
static qsl_status make_row_list(const uint32_t* worker_list, uint32_t R, RowList* rows) {
  if (R == 0 || R > 64) return QSL_ERR_INVALID_ARG;
  for (uint32_t q = 0; q < 64; ++q) rows->row[q] = q < R ? (worker_list ? worker_list[q] : q) : 0;
  for (uint32_t q = 0; q < R; ++q)
    for (uint32_t p = 0; p < q; ++p)
      if (rows->row[p] == rows->row[q]) return QSL_ERR_INVALID_ARG;
  return QSL_OK;
}

// The launches of the master line.  `dir` is room for R directories of `ndir` words, or null (then every message is
// searched whole); `nnz_hint` sizes the grids.
static qsl_status launch_aggregate(const DevCtx& c, hipStream_t st, uint32_t nnz_hint, uint32_t* dir, uint32_t ndir,
                                   const uint8_t* msg, const RowList& rows, uint32_t R, float scale, int accumulate,
                                   float* out) {
  if (c.K == c.d && (c.dense || !is_qsgd(c.quantizer))) {   // k = d and nothing dropped: every message lists every coordinate
    const uint32_t blocks = static_cast<uint32_t>(std::min<uint64_t>((c.d / 8 + BLOCK) / BLOCK, 1u << 16));   // two groups of four per thread
    k_aggregate_dense<<<dim3(blocks), BLOCK, 0, st>>>(c, msg, rows, R, scale, accumulate, out);
    QSL_HIP(hipGetLastError());
    return QSL_OK;
  }
  if (!accumulate) {
    const uint32_t blocks = static_cast<uint32_t>(std::min<uint64_t>((c.d + BLOCK * 4 - 1) / (BLOCK * 4), 1u << 16));
    k_fill_zero<<<dim3(blocks), BLOCK, 0, st>>>(out, c.d);
  }
  const bool by_ranges = R >= AGG_RANGES_MIN_R || (R >= AGG_RANGES_MIN_R_LONG && nnz_hint >= AGG_DIR_MIN);
  if (dir && by_ranges) {                           // many messages: a wave per 1024 coordinates, work linear in the entries
    uint32_t* dense_list = dir + 64ull * ndir;      // behind the 64 directories: a counter and up to ndir - 1 ranges
    k_msg_directory<<<dim3(std::min(2048u, (c.K + BLOCK - 1) / BLOCK), R), BLOCK, 0, st>>>(c, msg, rows, dir, ndir, dense_list);
    k_aggregate_ranges<<<dim3(ndir - 1), 64, 0, st>>>(c, msg, rows, R, scale, accumulate, out, dir, ndir, dense_list);
    k_aggregate_dense_ranges<<<dim3(std::min(AGG_DENSE_BLOCKS, ndir - 1)), 1024, 0, st>>>(c, msg, rows, R, scale, accumulate, out, dir,
                                                                                        ndir, dense_list);
    QSL_HIP(hipGetLastError());
    return QSL_OK;
  }
  if (R == 1 || nnz_hint < AGG_DIR_MIN) dir = nullptr;   // short messages are searched whole
  if (dir) {                                        // long messages: a thread per entry, searches narrowed by the directories
    k_msg_directory<<<dim3(std::min(2048u, (c.K + BLOCK - 1) / BLOCK), R), BLOCK, 0, st>>>(c, msg, rows, dir, ndir, nullptr);
    const uint32_t eb = std::min((c.K + BLOCK - 1) / BLOCK, std::max(4u, (nnz_hint + BLOCK - 1) / BLOCK));
    k_aggregate_entries<<<dim3(eb, R), BLOCK, 0, st>>>(c, msg, rows, R, scale, accumulate, out, dir, ndir);
  } else {                                          // short messages: 8 threads per entry, a block per expected tile of 32
    const uint32_t tiles = (c.K + AGG_ENTRIES - 1) / AGG_ENTRIES;
    const uint32_t agg_blocks = std::min(tiles, std::max(16u, (nnz_hint + AGG_ENTRIES - 1) / AGG_ENTRIES));
    k_aggregate<<<dim3(agg_blocks, R), BLOCK, 0, st>>>(c, msg, rows, R, scale, accumulate, out);
  }
  QSL_HIP(hipGetLastError());
  return QSL_OK;
}

extern "C" qsl_status qsl_aggregate(qsl_ctx* ctx, const uint8_t* msg, const uint32_t* worker_list, uint32_t R,
                                    float scale, int accumulate, float* out) {
  if (!ctx || !msg || !out) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(msg) & 7) || (reinterpret_cast<uintptr_t>(out) & 3)) return QSL_ERR_INVALID_ARG;
  RowList rows;
  const qsl_status st = make_row_list(worker_list, R, &rows);
  if (st != QSL_OK) return st;
  // the directories were allocated at qsl_create for operators whose messages are long
  return launch_aggregate(ctx->dc, ctx->stream, ctx->nnz_hint, ctx->agg_dir, ctx->agg_ndir, msg, rows, R, scale,
                          accumulate, out);
}

// ----------------------------------------------------------------------------------------------------
// the master line for callers that cannot allocate: the kernels' scratch is a fixed array of the library
// ----------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[QSL_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_STATIC_DEVICES = 64;
constexpr uint64_t STATIC_DIR_OFFSET = 256;       // bytes [0, 256): the status word; then the directories
void* g_scratch_ptr[MAX_STATIC_DEVICES];          // where `scratch` lies on each GPU (every GPU holds its own copy)
std::mutex g_scratch_mutex;

__global__ void k_clear_word(uint32_t* p) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *p = 0;
}

// the device address of `scratch` on the current GPU; in host code the array's name is not that address
qsl_status static_scratch(unsigned char** out) {
  int dev = -1;
  QSL_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_STATIC_DEVICES) return QSL_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    QSL_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return QSL_ERR_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
  return QSL_OK;
}
}  // namespace

extern "C" qsl_status qsl_aggregate_static(const qsl_config* cfg, void* hip_stream, const uint8_t* msg,
                                           const uint32_t* worker_list, uint32_t R, float scale, int accumulate,
                                           float* out) {
  uint64_t K64 = 0;
  if (!msg || !out) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(msg) & 7) || (reinterpret_cast<uintptr_t>(out) & 3)) return QSL_ERR_INVALID_ARG;
  qsl_status st = check_config(cfg, &K64);
  if (st != QSL_OK) return st;
  if (cfg->num_segments != 1) return QSL_ERR_UNSUPPORTED;     // segment tables would need device memory of their own
  RowList rows;
  st = make_row_list(worker_list, R, &rows);
  if (st != QSL_OK) return st;
  const WireDims wd = wire_dims(cfg, K64);
  if (wd.capacity / 4 > 0xFFFFFFFFull) return QSL_ERR_UNSUPPORTED;
  const uint32_t ndir = static_cast<uint32_t>(((cfg->d + (1u << AGG_DIR_SHIFT) - 1) >> AGG_DIR_SHIFT) + 1);
  const bool by_ranges = R >= AGG_RANGES_MIN_R || (R >= AGG_RANGES_MIN_R_LONG && wd.nnz_hint >= AGG_DIR_MIN);
  const bool want_dir = R > 1 && (wd.nnz_hint >= AGG_DIR_MIN || by_ranges);   // as launch_aggregate uses them
  // (the kernels for many messages keep a list of up to ndir ranges behind 64 directories)
  const uint64_t dir_rows = by_ranges ? 65 : R;
  if (want_dir && STATIC_DIR_OFFSET + 4ull * dir_rows * ndir > QSL_STATIC_SCRATCH_BYTES) return QSL_ERR_UNSUPPORTED;
  unsigned char* base = nullptr;
  st = static_scratch(&base);
  if (st != QSL_OK) return st;

  DevCtx c;
  memset(&c, 0, sizeof c);
  c.d = cfg->d; c.seed = cfg->seed; c.L = 1; c.K = static_cast<uint32_t>(K64);
  c.s = wd.s; c.w_idx = wd.w_idx; c.w_lev = wd.w_lev; c.w_val = wd.w_val;
  c.sparsifier = cfg->sparsifier; c.quantizer = cfg->quantizer;
  c.cap_words = static_cast<uint32_t>(wd.capacity / 4);
  c.status = reinterpret_cast<uint32_t*>(base);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // the array keeps what the last call left: the status word starts at zero (a kernel, not a memset node, so that
  // the call can be captured into a graph); the directories are written in full before they are read
  k_clear_word<<<dim3(1), 64, 0, stream>>>(c.status);
  uint32_t* dir = want_dir ? reinterpret_cast<uint32_t*>(base + STATIC_DIR_OFFSET) : nullptr;
  return launch_aggregate(c, stream, wd.nnz_hint, dir, ndir, msg, rows, R, scale, accumulate, out);
}

extern "C" qsl_status qsl_bits_sent(qsl_ctx* ctx, const uint8_t* msg, uint32_t R, uint64_t* bits_host) {
  if (!ctx || !msg || !bits_host || R == 0 || R > 1024) return QSL_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(msg) & 7) return QSL_ERR_INVALID_ARG;
  const DevCtx& c = ctx->dc;
  k_read_nnz<<<dim3((R + 255) / 256), 256, 0, ctx->stream>>>(c, msg, R, ctx->d_nnz_tmp);
  std::vector<uint32_t> nnz(R);
  QSL_HIP(hipMemcpyAsync(nnz.data(), ctx->d_nnz_tmp, 4ull * R, hipMemcpyDeviceToHost, ctx->stream));
  QSL_HIP(hipStreamSynchronize(ctx->stream));
  const bool counts = is_qsgd(c.quantizer) && c.L > 1 && !c.dense;
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
    o[1] = us[u].cand; o[2] = us[u].tau; o[3] = us[u].n_gt; o[4] = us[u].need; o[5] = us[u].path == PATH_FAST ? us[u].T_used : us[u].T;
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
