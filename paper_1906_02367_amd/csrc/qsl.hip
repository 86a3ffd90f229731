// qsl.hip -- kernels and C ABI of the compression hot path of Qsparse-local-SGD for gfx950.
//
// One synchronisation step of Algorithm 1 (arXiv:1906.02367) for a batch of R workers:
//   k_stream        v = m + Delta (worker line 1), written over the error memory, in ONE pass over
//                   HBM; coordinates whose rank key reaches a per-unit guess threshold are appended,
//                   in coordinate order, to a small candidate pool
//   k_sample*       the guess: a quantile of a strided sample of |m + Delta| (Top_k); for Rand_k the
//                   keys are uniform random words, so the guess is analytic
//   k_pool_hist,    exact radix selection of the k-th largest key (Section 2.2: Top_k / Rand_k)
//   k_v_hist,       among the candidates -- or, when a guess fails or a unit is too small/dense for
//   k_hist_scan     guessing, over the whole vector (the general path, always exact)
//   k_tile_count/scan/write   ordered compaction of the selected coordinates, ties to the lower index
//   k_norm*         exact ||v_S||_2^2 or ||v_S||_1 (proof of Lemma 1; Lemma 3 with m = 1)
//   k_quantize      QSGD levels (Definition 1, example 1) or signs (Definition 2); error update
//                   m <- v - g on the transmitted coordinates (Algorithm 1, worker line 2)
//   k_surv_*, k_pack    the packed message
//   k_aggregate     master line of Algorithm 1, atomic-free
//
// A "unit" is one (worker, segment) pair: the operator is applied independently to each unit
// (Corollary 1).  Rank key: Top_k: magnitude bits of v shifted left by one; Rand_k: the
// coordinate's random word of stream 0.  Larger key first, ties to the lower coordinate.
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

constexpr uint32_t CHUNK = 1024;           // coordinates one wave handles at a time: 4 x (64 lanes x 4)
constexpr uint32_t CHUNKS_PER_TILE = 16;   // a tile is the work of one 256-thread block
constexpr uint32_t TILE = CHUNK * CHUNKS_PER_TILE;
constexpr uint32_t BLOCK = 256;
constexpr uint32_t HBINS = 4096;           // radix digits: 12 + 12 + 8 bits of the 32-bit rank key
constexpr uint32_t ACC_SLOTS = 20;         // 32-bit digits of the exact accumulator
constexpr uint32_t NORM_TILE = 4096;
constexpr uint32_t QBLOCK = 256;           // block of the quantise / compact kernels
constexpr uint32_t SAMPLE_BLOCKS = 32;
constexpr uint32_t POOL_HIST_BLOCKS = 16;

enum : uint32_t { PATH_FAST = 0, PATH_GENERAL = 1, PATH_FALLBACK = 2 };

struct SegInfo {
  uint64_t start, size;
  uint64_t pool_off;    // first pool entry of this segment inside one worker's pool
  uint32_t k, koff;     // koff: first slot in the [K] selected arrays
  uint32_t tile_base, ntiles;
  uint32_t mode;        // PATH_FAST or PATH_GENERAL, decided on the host from (size, k)
  uint32_t pool_cap;
  uint32_t n_runs;      // sample: runs of 64 consecutive coordinates
  uint32_t r_s;         // sample rank that defines the guess
  uint32_t T_static;    // Rand_k: analytic guess
  uint32_t pad;
};

struct TileInfo { uint32_t seg, first_chunk, nchunks, pad; };
struct NormTile { uint32_t seg, first, count, pad; };

struct UnitState {
  uint32_t path, T, cand, overflow;
  uint32_t prefix, k_rem, tau, need;
  uint32_t n_gt, nnz, scale_bits, pad;
};

struct DevCtx {
  const SegInfo* segs; const TileInfo* tiles; const NormTile* ntiles; const uint32_t* fast_segs;
  UnitState* units;
  uint2* pool; uint64_t pool_stride;
  uint2* tile_rec;      // [R][NT]: (offset in the unit's pool, count) of the tile's candidates
  uint2* tile_cnt;      // [R][NT]: (#key > tau, #key == tau), then their exclusive prefix inside the unit
  uint32_t* hist;       // [U][HBINS]
  uint64_t* norm_acc;   // [U][ACC_SLOTS]
  uint32_t* sel_idx; uint32_t* sel_val; uint32_t* sel_code;   // [R][K]; code = level | neg << 31
  uint32_t* blk_cnt;    // [R][QB] survivors per quantise block, then exclusive prefix
  uint32_t* nnz_total;  // [R]
  uint32_t* surv_idx; uint32_t* surv_code;                    // [R][K]
  uint32_t* status; uint32_t* any_fallback;
  uint64_t d, seed;
  uint32_t L, K, NT, NNT, QB, nfast, s, w_idx, w_lev, w_val, sparsifier, quantizer, has_general, cap_words;
};

__device__ __forceinline__ uint32_t key_of_value(uint32_t vbits) { return (vbits & 0x7FFFFFFFu) << 1; }

template <int SPARS>
__device__ __forceinline__ uint32_t entry_key(uint2 e, const RandKey& rk) {
  return SPARS == QSL_TOPK ? key_of_value(e.y) : rand_word(rk, e.x);
}

// Find, scanning a 4096-bin histogram from its top, the bin in which the running count reaches
// `target` (1-based).  1024 threads.  Returns the bin; *above = count in the bins above it.
// If the histogram holds fewer than `target` entries, returns bin 0 with *above = total - hist[0].
__device__ uint32_t find_from_top(const uint32_t* hist, uint32_t target, uint32_t* above, uint64_t* scratch,
                                  uint32_t* result) {
  const uint32_t t = threadIdx.x;                 // thread t owns bins 4095-4t .. 4092-4t (top first)
  uint32_t h[4]; uint32_t sum = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) { h[j] = hist[HBINS - 1 - (4 * t + j)]; sum += h[j]; }
  uint64_t total;
  const uint64_t before = block_exclusive_scan64(sum, scratch, &total);
  if (t == 0) { result[0] = 0; result[1] = static_cast<uint32_t>(total) - hist[0]; }
  __syncthreads();
  if (before < target && before + sum >= target) {
    uint32_t cum = static_cast<uint32_t>(before);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (cum + h[j] >= target) { result[0] = HBINS - 1 - (4 * t + j); result[1] = cum; break; }
      cum += h[j];
    }
  }
  __syncthreads();
  *above = result[1];
  return result[0];
}

// ------------------------------------------------------------------------------------------------
// per-call initialisation
// ------------------------------------------------------------------------------------------------
__global__ void k_init(DevCtx c, uint32_t R) {
  const uint64_t gid = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  const uint32_t U = R * c.L;
  for (uint64_t i = gid; i < U; i += stride) {
    const SegInfo& sg = c.segs[i % c.L];
    UnitState u;
    u.path = sg.mode; u.T = sg.mode == PATH_FAST ? sg.T_static : 0xFFFFFFFFu; u.cand = 0; u.overflow = 0;
    u.prefix = 0; u.k_rem = sg.k; u.tau = 0; u.need = 0; u.n_gt = 0; u.nnz = 0; u.scale_bits = 0; u.pad = 0;
    c.units[i] = u;
  }
  for (uint64_t i = gid; i < static_cast<uint64_t>(U) * HBINS; i += stride) c.hist[i] = 0;
  for (uint64_t i = gid; i < static_cast<uint64_t>(U) * ACC_SLOTS; i += stride) c.norm_acc[i] = 0;
  if (gid == 0) *c.any_fallback = 0;
}

// ------------------------------------------------------------------------------------------------
// the guess for Top_k: histogram of the rank keys of a strided sample of v = m + Delta
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_sample(DevCtx c, const float* m, const float* delta) {
  __shared__ uint32_t lh[HBINS];
  const uint32_t seg = c.fast_segs[blockIdx.y], w = blockIdx.z;
  const SegInfo sg = c.segs[seg];
  for (uint32_t i = threadIdx.x; i < HBINS; i += BLOCK) lh[i] = 0;
  __syncthreads();
  const uint64_t row = static_cast<uint64_t>(w) * c.d + sg.start;
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  for (uint32_t run = blockIdx.x * 4 + wave; run < sg.n_runs; run += SAMPLE_BLOCKS * 4) {
    // run start: floor(run * size / n_runs); size < 2^32 and run < 2^32, so the product fits 64 bits
    const uint64_t pos = static_cast<uint64_t>(run) * sg.size / sg.n_runs + lane;
    if (pos < sg.size) {
      const float v = m[row + pos] + delta[row + pos];
      atomicAdd(&lh[key_of_value(__float_as_uint(v)) >> 20], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = c.hist + (static_cast<uint64_t>(w) * c.L + seg) * HBINS;
  for (uint32_t i = threadIdx.x; i < HBINS; i += BLOCK)
    if (lh[i]) atomicAdd(&gh[i], lh[i]);
}

__global__ __launch_bounds__(1024) void k_sample_scan(DevCtx c) {
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[2];
  const uint32_t seg = c.fast_segs[blockIdx.x], w = blockIdx.y;
  const SegInfo& sg = c.segs[seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
  uint32_t* gh = c.hist + u * HBINS;
  uint32_t above;
  const uint32_t bin = find_from_top(gh, sg.r_s, &above, scratch, result);
  if (threadIdx.x == 0) c.units[u].T = bin << 20;      // lower edge of the bin
  for (uint32_t i = threadIdx.x; i < HBINS; i += 1024) gh[i] = 0;
}

// ------------------------------------------------------------------------------------------------
// the streaming pass
// ------------------------------------------------------------------------------------------------
template <int SPARS>
__global__ __launch_bounds__(BLOCK) void k_stream(DevCtx c, const float* m,
                                                  const float* delta, float* m_out, uint32_t worker0,
                                                  uint64_t round) {
  __shared__ uint32_t s_cnt[CHUNKS_PER_TILE];
  __shared__ uint32_t s_base[CHUNKS_PER_TILE + 1];
  const TileInfo ti = c.tiles[blockIdx.x];
  const uint32_t w = blockIdx.y;
  const SegInfo sg = c.segs[ti.seg];
  UnitState* us = &c.units[static_cast<uint64_t>(w) * c.L + ti.seg];
  const bool collect = us->path == PATH_FAST;
  const uint32_t T = us->T;
  const uint64_t row = static_cast<uint64_t>(w) * c.d + sg.start;
  const float* mp = m + row;
  const float* dp = delta + row;
  float* op = m_out + row;
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  uint32_t pmask[4] = {0, 0, 0, 0};
  bool nonfinite = false;

#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t lc = q * 4 + wave;
    uint32_t pm = 0;
    if (lc < ti.nchunks) {
      const uint64_t cb = static_cast<uint64_t>(ti.first_chunk + lc) * CHUNK;   // segment-local
      const uint64_t left = sg.size - cb;
      if (left >= CHUNK) {
        f4u a[4], b[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint64_t e = cb + t * 256 + lane * 4;
          a[t] = *reinterpret_cast<const f4u*>(mp + e);
          b[t] = *reinterpret_cast<const f4u*>(dp + e);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint64_t e = cb + t * 256 + lane * 4;
          const f4u v = a[t] + b[t];
          *reinterpret_cast<f4u*>(op + e) = v;
          Words4 rw;
          if (SPARS == QSL_RANDK) rw = rand_words4(rk, static_cast<uint32_t>(sg.start + e));
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t bits = __float_as_uint(v[j]);
            nonfinite |= (bits & 0x7FFFFFFFu) >= 0x7F800000u;
            const uint32_t key = SPARS == QSL_TOPK ? key_of_value(bits) : rw.w[j];
            pm |= (key >= T ? 1u : 0u) << (t * 4 + j);
          }
        }
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint64_t e = cb + t * 256 + lane * 4 + j;
            if (e < sg.size) {
              const float v = mp[e] + dp[e];
              op[e] = v;
              const uint32_t bits = __float_as_uint(v);
              nonfinite |= (bits & 0x7FFFFFFFu) >= 0x7F800000u;
              const uint32_t key = SPARS == QSL_TOPK ? key_of_value(bits)
                                                     : rand_word(rk, static_cast<uint32_t>(sg.start + e));
              pm |= (key >= T ? 1u : 0u) << (t * 4 + j);
            }
          }
        }
      }
      if (!collect) pm = 0;
    }
    pmask[q] = pm;
    const uint32_t cnt = wave_sum(__popc(pm));
    if (lane == 0) s_cnt[lc] = cnt;
  }
  if (__ballot(nonfinite) != 0 && lane == 0) atomicOr(c.status, 1u);
  if (!collect) return;                           // uniform over the block

  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t run = 0;
    for (uint32_t i = 0; i < CHUNKS_PER_TILE; ++i) { s_base[i] = run; run += s_cnt[i]; }
    uint32_t off = 0;
    if (run) {
      off = atomicAdd(&us->cand, run);
      if (off > sg.pool_cap || run > sg.pool_cap - off) { us->overflow = 1; off = 0xFFFFFFFFu; }
    }
    s_base[CHUNKS_PER_TILE] = off;
    c.tile_rec[static_cast<uint64_t>(w) * c.NT + blockIdx.x] = make_uint2(off == 0xFFFFFFFFu ? 0u : off,
                                                                          off == 0xFFFFFFFFu ? 0u : run);
  }
  __syncthreads();
  const uint32_t off = s_base[CHUNKS_PER_TILE];
  if (off == 0xFFFFFFFFu) return;
  uint2* pool = c.pool + static_cast<uint64_t>(w) * c.pool_stride + sg.pool_off + off;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t pm = pmask[q];
    if (__ballot(pm != 0) == 0) continue;         // wave-uniform
    const uint32_t lc = q * 4 + wave;
    const uint64_t cb = static_cast<uint64_t>(ti.first_chunk + lc) * CHUNK;
    uint32_t base = s_base[lc];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint32_t nib = (pm >> (t * 4)) & 0xFu;
      if (__ballot(nib != 0) == 0) continue;      // wave-uniform
      uint32_t before = 0, total = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint64_t bal = __ballot((nib >> j) & 1u);
        before += popc_below(bal);
        total += __popcll(bal);
      }
      uint32_t pos = base + before;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if ((nib >> j) & 1u) {
          const uint64_t e = cb + t * 256 + lane * 4 + j;
          pool[pos++] = make_uint2(static_cast<uint32_t>(sg.start + e), __float_as_uint(op[e]));
        }
      }
      base += total;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// validation of the guess; radix selection
// ------------------------------------------------------------------------------------------------
__global__ void k_validate(DevCtx c, uint32_t U) {
  const uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= U) return;
  UnitState* us = &c.units[u];
  if (us->path == PATH_FAST && (us->overflow || us->cand < c.segs[u % c.L].k)) {
    us->path = PATH_FALLBACK;
    atomicOr(c.any_fallback, 1u);
  }
}

template <int LEVEL>
__device__ __forceinline__ bool level_bin(uint32_t key, uint32_t prefix, uint32_t* bin) {
  if (LEVEL == 0) { *bin = key >> 20; return true; }
  if (LEVEL == 1) { *bin = (key >> 8) & 0xFFFu; return (key >> 20) == (prefix >> 20); }
  *bin = key & 0xFFu; return (key >> 8) == (prefix >> 8);
}

template <int LEVEL, int SPARS>
__global__ __launch_bounds__(BLOCK) void k_pool_hist(DevCtx c, uint32_t worker0, uint64_t round) {
  __shared__ uint32_t lh[HBINS];
  const uint32_t seg = c.fast_segs[blockIdx.y], w = blockIdx.z;
  const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
  const UnitState us = c.units[u];
  if (us.path != PATH_FAST) return;
  const SegInfo& sg = c.segs[seg];
  for (uint32_t i = threadIdx.x; i < HBINS; i += BLOCK) lh[i] = 0;
  __syncthreads();
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint2* pool = c.pool + static_cast<uint64_t>(w) * c.pool_stride + sg.pool_off;
  for (uint32_t e = blockIdx.x * BLOCK + threadIdx.x; e < us.cand; e += POOL_HIST_BLOCKS * BLOCK) {
    uint32_t bin;
    if (level_bin<LEVEL>(entry_key<SPARS>(pool[e], rk), us.prefix, &bin)) atomicAdd(&lh[bin], 1u);
  }
  __syncthreads();
  uint32_t* gh = c.hist + u * HBINS;
  for (uint32_t i = threadIdx.x; i < HBINS; i += BLOCK)
    if (lh[i]) atomicAdd(&gh[i], lh[i]);
}

// rank key of a coordinate in the general path: from v (already written to m_out) or its random word
template <int SPARS>
__device__ __forceinline__ uint32_t coord_key(const float* vp, uint64_t e, uint64_t start, const RandKey& rk) {
  return SPARS == QSL_TOPK ? key_of_value(__float_as_uint(vp[e])) : rand_word(rk, static_cast<uint32_t>(start + e));
}

template <int LEVEL, int SPARS>
__global__ __launch_bounds__(BLOCK) void k_v_hist(DevCtx c, const float* v, uint32_t worker0, uint64_t round) {
  __shared__ uint32_t lh[HBINS];
  if (!c.has_general && !*c.any_fallback) return;
  const uint32_t w = blockIdx.y;
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  for (uint32_t t = blockIdx.x; t < c.NT; t += gridDim.x) {
    const TileInfo ti = c.tiles[t];
    const uint64_t u = static_cast<uint64_t>(w) * c.L + ti.seg;
    const UnitState us = c.units[u];
    if (us.path == PATH_FAST) continue;
    const SegInfo& sg = c.segs[ti.seg];
    for (uint32_t i = threadIdx.x; i < HBINS; i += BLOCK) lh[i] = 0;
    __syncthreads();
    const float* vp = v + static_cast<uint64_t>(w) * c.d + sg.start;
    const uint64_t lo = static_cast<uint64_t>(ti.first_chunk) * CHUNK;
    const uint64_t hi = std::min<uint64_t>(sg.size, lo + static_cast<uint64_t>(ti.nchunks) * CHUNK);
    for (uint64_t e = lo + threadIdx.x; e < hi; e += BLOCK) {
      uint32_t bin;
      if (level_bin<LEVEL>(coord_key<SPARS>(vp, e, sg.start, rk), us.prefix, &bin)) atomicAdd(&lh[bin], 1u);
    }
    __syncthreads();
    uint32_t* gh = c.hist + u * HBINS;
    for (uint32_t i = threadIdx.x; i < HBINS; i += BLOCK)
      if (lh[i]) atomicAdd(&gh[i], lh[i]);
    __syncthreads();
  }
}

template <int LEVEL>
__global__ __launch_bounds__(1024) void k_hist_scan(DevCtx c) {
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[2];
  const uint64_t u = static_cast<uint64_t>(blockIdx.y) * c.L + blockIdx.x;
  UnitState* us = &c.units[u];
  uint32_t* gh = c.hist + u * HBINS;
  uint32_t above;
  const uint32_t k_rem = us->k_rem;
  const uint32_t bin = find_from_top(gh, k_rem, &above, scratch, result);
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t shift = LEVEL == 0 ? 20 : LEVEL == 1 ? 8 : 0;
    const uint32_t prefix = us->prefix | (bin << shift);
    us->prefix = prefix;
    us->k_rem = k_rem - above;
    if (LEVEL == 2) {
      us->tau = prefix;
      us->need = k_rem - above;                       // how many coordinates with key == tau are kept
      us->n_gt = c.segs[blockIdx.x].k - (k_rem - above);
    }
  }
  for (uint32_t i = threadIdx.x; i < HBINS; i += 1024) gh[i] = 0;
}

// ------------------------------------------------------------------------------------------------
// ordered compaction of the selected coordinates
// ------------------------------------------------------------------------------------------------
template <int SPARS>
__global__ __launch_bounds__(BLOCK) void k_tile_count(DevCtx c, const float* v, uint32_t worker0, uint64_t round) {
  __shared__ uint32_t s_gt[4], s_eq[4];
  const TileInfo ti = c.tiles[blockIdx.x];
  const uint32_t w = blockIdx.y;
  const uint64_t u = static_cast<uint64_t>(w) * c.L + ti.seg;
  const UnitState us = c.units[u];
  const SegInfo& sg = c.segs[ti.seg];
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  uint2* out = &c.tile_cnt[static_cast<uint64_t>(w) * c.NT + blockIdx.x];
  uint32_t gt = 0, eq = 0;
  if (us.path == PATH_FAST) {
    if (wave != 0) return;
    const uint2 rec = c.tile_rec[static_cast<uint64_t>(w) * c.NT + blockIdx.x];
    const uint2* pool = c.pool + static_cast<uint64_t>(w) * c.pool_stride + sg.pool_off + rec.x;
    for (uint32_t e = lane; e < rec.y; e += WAVE) {
      const uint32_t key = entry_key<SPARS>(pool[e], rk);
      gt += key > us.tau; eq += key == us.tau;
    }
    gt = wave_sum(gt); eq = wave_sum(eq);
    if (lane == 0) *out = make_uint2(gt, eq);
    return;
  }
  const float* vp = v + static_cast<uint64_t>(w) * c.d + sg.start;
  const uint64_t lo = static_cast<uint64_t>(ti.first_chunk) * CHUNK;
  const uint64_t hi = std::min<uint64_t>(sg.size, lo + static_cast<uint64_t>(ti.nchunks) * CHUNK);
  for (uint64_t e = lo + threadIdx.x; e < hi; e += BLOCK) {
    const uint32_t key = coord_key<SPARS>(vp, e, sg.start, rk);
    gt += key > us.tau; eq += key == us.tau;
  }
  gt = wave_sum(gt); eq = wave_sum(eq);
  if (lane == 0) { s_gt[wave] = gt; s_eq[wave] = eq; }
  __syncthreads();
  if (threadIdx.x == 0) *out = make_uint2(s_gt[0] + s_gt[1] + s_gt[2] + s_gt[3], s_eq[0] + s_eq[1] + s_eq[2] + s_eq[3]);
}

// exclusive prefix of the (greater, equal) tile counts inside each unit; one block per unit
__global__ __launch_bounds__(1024) void k_tile_scan(DevCtx c) {
  __shared__ uint64_t scratch[17];
  const SegInfo& sg = c.segs[blockIdx.x];
  uint2* cnt = c.tile_cnt + static_cast<uint64_t>(blockIdx.y) * c.NT + sg.tile_base;
  uint64_t carry = 0;
  for (uint32_t base = 0; base < sg.ntiles; base += 1024) {
    const uint32_t i = base + threadIdx.x;
    uint64_t x = 0;
    if (i < sg.ntiles) { const uint2 p = cnt[i]; x = (static_cast<uint64_t>(p.y) << 32) | p.x; }
    uint64_t total;
    const uint64_t ex = block_exclusive_scan64(x, scratch, &total) + carry;
    if (i < sg.ntiles) cnt[i] = make_uint2(static_cast<uint32_t>(ex), static_cast<uint32_t>(ex >> 32));
    carry += total;
  }
}

template <int SPARS>
__global__ __launch_bounds__(BLOCK) void k_tile_write(DevCtx c, const float* v, uint32_t worker0, uint64_t round) {
  __shared__ uint32_t s_gt[CHUNKS_PER_TILE + 1], s_eq[CHUNKS_PER_TILE + 1];
  const TileInfo ti = c.tiles[blockIdx.x];
  const uint32_t w = blockIdx.y;
  const uint64_t u = static_cast<uint64_t>(w) * c.L + ti.seg;
  const UnitState us = c.units[u];
  const SegInfo& sg = c.segs[ti.seg];
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint2 base = c.tile_cnt[static_cast<uint64_t>(w) * c.NT + blockIdx.x];
  uint32_t* oi = c.sel_idx + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint32_t* ov = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff;
  if (us.path == PATH_FAST) {
    if (wave != 0) return;
    const uint2 rec = c.tile_rec[static_cast<uint64_t>(w) * c.NT + blockIdx.x];
    const uint2* pool = c.pool + static_cast<uint64_t>(w) * c.pool_stride + sg.pool_off + rec.x;
    uint32_t gt_before = base.x, eq_before = base.y;
    for (uint32_t e0 = 0; e0 < rec.y; e0 += WAVE) {
      const uint32_t e = e0 + lane;
      uint2 ent = make_uint2(0, 0);
      bool is_gt = false, is_eq = false;
      if (e < rec.y) {
        ent = pool[e];
        const uint32_t key = entry_key<SPARS>(ent, rk);
        is_gt = key > us.tau; is_eq = key == us.tau;
      }
      const uint64_t bg = __ballot(is_gt), be = __ballot(is_eq);
      const uint32_t my_gt = gt_before + popc_below(bg), my_eq = eq_before + popc_below(be);
      if (is_gt || (is_eq && my_eq < us.need)) {
        const uint32_t pos = my_gt + min(my_eq, us.need);
        oi[pos] = ent.x; ov[pos] = ent.y;
      }
      gt_before += __popcll(bg); eq_before += __popcll(be);
    }
    return;
  }
  // general path: per-chunk counts first, so that every wave knows where its chunks start
  const float* vp = v + static_cast<uint64_t>(w) * c.d + sg.start;
  for (uint32_t lc = wave; lc < CHUNKS_PER_TILE; lc += 4) {
    uint32_t gt = 0, eq = 0;
    if (lc < ti.nchunks) {
      const uint64_t cb = static_cast<uint64_t>(ti.first_chunk + lc) * CHUNK;
      for (uint32_t j = lane; j < CHUNK; j += WAVE) {
        const uint64_t e = cb + j;
        if (e < sg.size) {
          const uint32_t key = coord_key<SPARS>(vp, e, sg.start, rk);
          gt += key > us.tau; eq += key == us.tau;
        }
      }
    }
    gt = wave_sum(gt); eq = wave_sum(eq);
    if (lane == 0) { s_gt[lc] = gt; s_eq[lc] = eq; }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t rg = base.x, re = base.y;
    for (uint32_t i = 0; i < CHUNKS_PER_TILE; ++i) {
      const uint32_t g = s_gt[i], q = s_eq[i];
      s_gt[i] = rg; s_eq[i] = re; rg += g; re += q;
    }
  }
  __syncthreads();
  for (uint32_t lc = wave; lc < ti.nchunks; lc += 4) {
    const uint64_t cb = static_cast<uint64_t>(ti.first_chunk + lc) * CHUNK;
    uint32_t gt_before = s_gt[lc], eq_before = s_eq[lc];
    for (uint32_t j0 = 0; j0 < CHUNK; j0 += WAVE) {
      const uint64_t e = cb + j0 + lane;
      bool is_gt = false, is_eq = false;
      uint32_t bits = 0;
      if (e < sg.size) {
        bits = __float_as_uint(vp[e]);
        const uint32_t key = SPARS == QSL_TOPK ? key_of_value(bits) : rand_word(rk, static_cast<uint32_t>(sg.start + e));
        is_gt = key > us.tau; is_eq = key == us.tau;
      }
      const uint64_t bg = __ballot(is_gt), be = __ballot(is_eq);
      const uint32_t my_gt = gt_before + popc_below(bg), my_eq = eq_before + popc_below(be);
      if (is_gt || (is_eq && my_eq < us.need)) {
        const uint32_t pos = my_gt + min(my_eq, us.need);
        oi[pos] = static_cast<uint32_t>(sg.start + e); ov[pos] = bits;
      }
      gt_before += __popcll(bg); eq_before += __popcll(be);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// exact norms: every |v| (or v^2) is an integer multiple of 2^-149 (2^-298); its 32-bit digits are
// added into 64-bit counters, integer addition commutes, so any schedule gives the same sum
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_norm(DevCtx c) {
  __shared__ uint64_t acc[BLOCK * (ACC_SLOTS + 1)];
  const NormTile nt = c.ntiles[blockIdx.x];
  const uint32_t w = blockIdx.y;
  const SegInfo& sg = c.segs[nt.seg];
  uint64_t* mine = acc + threadIdx.x * (ACC_SLOTS + 1);
#pragma unroll
  for (uint32_t i = 0; i < ACC_SLOTS; ++i) mine[i] = 0;
  const uint32_t* val = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff + nt.first;
  for (uint32_t j = threadIdx.x; j < nt.count; j += BLOCK) {
    const uint32_t ab = val[j] & 0x7FFFFFFFu;
    const uint32_t ex = ab >> 23, frac = ab & 0x7FFFFFu;
    const uint32_t M = ex ? (frac | 0x800000u) : frac;       // |v| = M * 2^(max(ex,1) - 150)
    const uint32_t e1 = ex ? ex : 1u;
    if (M == 0) continue;
    if (c.quantizer == QSL_QSGD) {
      const uint64_t sq = static_cast<uint64_t>(M) * M;       // < 2^48;  v^2 = sq * 2^(2 e1 - 300)
      const uint32_t p = 2u * e1 - 2u;                        // bit position above 2^-298
      const uint32_t q = p >> 5, r = p & 31u;
      const uint64_t lo = sq << r;                            // low 64 bits of sq * 2^r  (r <= 30)
      const uint64_t hi = r ? (sq >> (64 - r)) : 0;
      mine[q] += lo & 0xFFFFFFFFu; mine[q + 1] += lo >> 32; mine[q + 2] += hi;
    } else {
      const uint32_t p = e1 - 1u;                             // bit position above 2^-149
      const uint32_t q = p >> 5, r = p & 31u;
      const uint64_t sh = static_cast<uint64_t>(M) << r;      // < 2^55
      mine[q] += sh & 0xFFFFFFFFu; mine[q + 1] += sh >> 32;
    }
  }
  __syncthreads();
  if (threadIdx.x < ACC_SLOTS) {
    uint64_t sum = 0;
    for (uint32_t t = 0; t < BLOCK; ++t) sum += acc[t * (ACC_SLOTS + 1) + threadIdx.x];
    if (sum) atomicAdd(reinterpret_cast<unsigned long long*>(c.norm_acc + (static_cast<uint64_t>(w) * c.L + nt.seg) * ACC_SLOTS + threadIdx.x),
                       static_cast<unsigned long long>(sum));
  }
}

// digits -> one correctly rounded double -> the fp32 scale of the unit
__global__ void k_norm_finalize(DevCtx c, uint32_t U) {
  const uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= U) return;
  const uint64_t* a = c.norm_acc + static_cast<uint64_t>(u) * ACC_SLOTS;
  uint32_t dig[ACC_SLOTS + 1];
  uint64_t carry = 0;
  for (uint32_t i = 0; i < ACC_SLOTS; ++i) { const uint64_t t = a[i] + carry; dig[i] = static_cast<uint32_t>(t); carry = t >> 32; }
  dig[ACC_SLOTS] = static_cast<uint32_t>(carry);
  int top = -1;
  for (int i = ACC_SLOTS; i >= 0; --i) if (dig[i]) { top = i * 32 + 31 - __clz(dig[i]); break; }
  double S = 0.0;
  if (top >= 0) {
    const int low = top - 52;                 // last kept bit
    uint64_t mant = 0;
    for (int b = top; b >= (low > 0 ? low : 0); --b) mant = (mant << 1) | ((dig[b >> 5] >> (b & 31)) & 1u);
    int e2 = low > 0 ? low : 0;
    if (low > 0) {
      const uint32_t guard = (dig[(low - 1) >> 5] >> ((low - 1) & 31)) & 1u;
      bool sticky = false;
      for (int b = 0; b < low - 1; ++b) sticky |= (dig[b >> 5] >> (b & 31)) & 1u;
      if (guard && (sticky || (mant & 1u))) mant += 1;
    }
    S = ldexp(static_cast<double>(mant), e2 + (c.quantizer == QSL_QSGD ? -298 : -149));
  }
  float scale;
  if (c.quantizer == QSL_QSGD) scale = static_cast<float>(sqrt(S));
  else scale = static_cast<float>(S / static_cast<double>(c.segs[u % c.L].k));
  c.units[u].scale_bits = __float_as_uint(scale);
}

// ------------------------------------------------------------------------------------------------
// quantise, error update, message
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t seg_of_slot(const DevCtx& c, uint32_t j) {   // segment owning slot j of [K]
  uint32_t lo = 0, hi = c.L;
  while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (c.segs[mid].koff <= j) lo = mid; else hi = mid; }
  return lo;
}
__device__ __forceinline__ uint32_t seg_of_coord(const DevCtx& c, uint32_t i) {
  uint32_t lo = 0, hi = c.L;
  while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (c.segs[mid].start <= i) lo = mid; else hi = mid; }
  return lo;
}

__device__ __forceinline__ float qsgd_value(float N, uint32_t level, uint32_t s, bool neg) {
  const float prod = N * static_cast<float>(level);
  const float mag = prod / static_cast<float>(s);
  return neg ? -mag : mag;
}

__global__ __launch_bounds__(QBLOCK) void k_quantize(DevCtx c, float* m_out, uint32_t worker0, uint64_t round,
                                                     uint32_t* dbg_idx, uint16_t* dbg_level) {
  __shared__ uint32_t s_w[QBLOCK / 64];
  const uint32_t w = blockIdx.y;
  const uint32_t j = blockIdx.x * QBLOCK + threadIdx.x;
  uint32_t sent = 0;
  if (j < c.K) {
    const uint32_t seg = c.L == 1 ? 0u : seg_of_slot(c, j);
    const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
    const uint64_t slot = static_cast<uint64_t>(w) * c.K + j;
    const uint32_t idx = c.sel_idx[slot], bits = c.sel_val[slot];
    const float scale = __uint_as_float(c.units[u].scale_bits);
    const float v = __uint_as_float(bits);
    const bool neg = v < 0.0f;
    uint32_t level;
    float g;
    if (c.quantizer == QSL_QSGD) {
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
      g = qsgd_value(scale, level, c.s, neg);
    } else {
      level = 1;
      g = neg ? -scale : scale;
    }
    sent = level != 0;
    c.sel_code[slot] = level | (neg ? 0x80000000u : 0u);
    if (sent) {
      if (idx < c.d) m_out[static_cast<uint64_t>(w) * c.d + idx] = v - g;
      else atomicOr(c.status, 2u);                       // cannot happen: a selected slot was never written
      if (c.quantizer == QSL_QSGD && c.L > 1) atomicAdd(&c.units[u].nnz, 1u);
    }
    if (dbg_idx) dbg_idx[slot] = idx;
    if (dbg_level) dbg_level[slot] = static_cast<uint16_t>(level);
  }
  const uint32_t wc = __popcll(__ballot(sent));
  if (lane_id() == 0) s_w[threadIdx.x >> 6] = wc;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
    for (uint32_t i = 0; i < QBLOCK / 64; ++i) t += s_w[i];
    c.blk_cnt[static_cast<uint64_t>(w) * c.QB + blockIdx.x] = t;
  }
}

__global__ __launch_bounds__(1024) void k_surv_scan(DevCtx c) {
  __shared__ uint64_t scratch[17];
  uint32_t* cnt = c.blk_cnt + static_cast<uint64_t>(blockIdx.x) * c.QB;
  uint64_t carry = 0;
  for (uint32_t base = 0; base < c.QB; base += 1024) {
    const uint32_t i = base + threadIdx.x;
    const uint64_t x = i < c.QB ? cnt[i] : 0;
    uint64_t total;
    const uint64_t ex = block_exclusive_scan64(x, scratch, &total) + carry;
    if (i < c.QB) cnt[i] = static_cast<uint32_t>(ex);
    carry += total;
  }
  if (threadIdx.x == 0) c.nnz_total[blockIdx.x] = static_cast<uint32_t>(carry);
}

__global__ __launch_bounds__(QBLOCK) void k_surv_compact(DevCtx c) {
  __shared__ uint32_t s_w[QBLOCK / 64];
  const uint32_t w = blockIdx.y;
  const uint32_t j = blockIdx.x * QBLOCK + threadIdx.x;
  uint32_t code = 0;
  const uint64_t slot = static_cast<uint64_t>(w) * c.K + j;
  if (j < c.K) code = c.sel_code[slot];
  const bool sent = (code & 0x7FFFFFFFu) != 0;
  const uint64_t bal = __ballot(sent);
  if (lane_id() == 0) s_w[threadIdx.x >> 6] = __popcll(bal);
  __syncthreads();
  uint32_t pos = c.blk_cnt[static_cast<uint64_t>(w) * c.QB + blockIdx.x] + popc_below(bal);
  for (uint32_t i = 0; i < (threadIdx.x >> 6); ++i) pos += s_w[i];
  if (sent) {
    const uint32_t level = code & 0x7FFFFFFFu, neg = code >> 31;
    c.surv_idx[static_cast<uint64_t>(w) * c.K + pos] = c.sel_idx[slot];
    c.surv_code[static_cast<uint64_t>(w) * c.K + pos] = c.quantizer == QSL_QSGD ? ((level - 1u) | (neg << c.w_lev)) : neg;
  }
}

// one thread per 32-bit word of the message: it gathers the fields that overlap its word
__device__ __forceinline__ uint32_t gather_word(const uint32_t* arr, uint64_t n, uint32_t width, uint64_t word) {
  if (width == 0) return 0;
  const uint64_t b0 = word * 32;
  uint32_t out = 0;
  for (uint64_t e = b0 / width; e < n && e * width < b0 + 32; ++e) {
    const int64_t sh = static_cast<int64_t>(e * width) - static_cast<int64_t>(b0);
    const uint32_t f = arr[e];
    out |= sh >= 0 ? (f << sh) : (f >> (-sh));
  }
  return out;
}

__global__ __launch_bounds__(BLOCK) void k_pack(DevCtx c, uint8_t* msg, uint64_t* msg_bits) {
  const uint32_t w = blockIdx.y;
  const uint64_t q = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x;
  if (q >= c.cap_words) return;
  const uint64_t nnz = c.nnz_total[w];
  const bool counts = c.quantizer == QSL_QSGD && c.L > 1;
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
  const bool counts = c.quantizer == QSL_QSGD && c.L > 1;
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
  if (c.quantizer == QSL_QSGD) {
    const uint32_t level = (code & ((1u << c.w_lev) - 1u)) + 1u;
    return qsgd_value(scale, level, c.s, (code >> c.w_lev) & 1u);
  }
  return code ? -scale : scale;
}
// position of coordinate idx in the message, or -1
__device__ __forceinline__ int64_t msg_find(const DevCtx& c, const MsgView& v, uint32_t idx) {
  uint32_t lo = 0, hi = v.nnz;
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    const uint32_t x = msg_index(c, v, mid);
    if (x == idx) return mid;
    if (x < idx) lo = mid + 1; else hi = mid;
  }
  return -1;
}

__global__ __launch_bounds__(BLOCK) void k_add_rows(float* m, const float* delta, uint64_t n) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * BLOCK * 4;
  for (uint64_t i = (static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 4 <= n) {
      const f4u a = *reinterpret_cast<const f4u*>(m + i), b = *reinterpret_cast<const f4u*>(delta + i);
      *reinterpret_cast<f4u*>(m + i) = a + b;
    } else {
      for (uint64_t j = i; j < n; ++j) m[j] = m[j] + delta[j];
    }
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

__global__ __launch_bounds__(BLOCK) void k_fill_zero(float* out, uint64_t n) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * BLOCK * 4;
  const f4u z = {0.f, 0.f, 0.f, 0.f};
  for (uint64_t i = (static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 4 <= n) *reinterpret_cast<f4u*>(out + i) = z;
    else for (uint64_t j = i; j < n; ++j) out[j] = 0.f;
  }
}

struct RowList { uint32_t row[64]; };

// Thread (q, j) owns entry j of the q-th listed message.  It writes out[idx] only if no earlier
// listed message holds idx; it then adds the later messages' values in list order: no atomics,
// one writer per coordinate, a fixed summation order.
__global__ __launch_bounds__(BLOCK) void k_aggregate(DevCtx c, const uint8_t* msg, RowList rows, uint32_t R,
                                                     float scale, int accumulate, float* out) {
  const uint32_t q = blockIdx.y;
  const MsgView mine = view_msg(c, msg, rows.row[q]);
  const uint32_t j = blockIdx.x * BLOCK + threadIdx.x;
  if (j >= mine.nnz) return;
  const uint32_t idx = msg_index(c, mine, j);
  if (idx >= c.d) { atomicOr(c.status, 4u); return; }   // malformed message
  for (uint32_t p = 0; p < q; ++p) {
    const MsgView other = view_msg(c, msg, rows.row[p]);
    if (msg_find(c, other, idx) >= 0) return;
  }
  float acc = msg_value(c, mine, j, idx);
  for (uint32_t p = q + 1; p < R; ++p) {
    const MsgView other = view_msg(c, msg, rows.row[p]);
    const int64_t pos = msg_find(c, other, idx);
    if (pos >= 0) acc = acc + msg_value(c, other, static_cast<uint32_t>(pos), idx);
  }
  const float term = scale * acc;
  out[idx] = accumulate ? out[idx] + term : term;
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
  void* slab;                 // one allocation holding every scratch array
  uint32_t Rmax;
  uint32_t last_R;
  size_t capacity;
  uint32_t* h_status;         // pinned
  uint32_t* d_nnz_tmp;
  int timing;
  std::vector<hipEvent_t> ev;
  size_t ev_used;
  double ev_ms;
  uint32_t ev_launches;
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

extern "C" qsl_status qsl_create(qsl_ctx** out, const qsl_config* cfg, void* hip_stream) {
  if (!out || !cfg || !cfg->seg_offset || !cfg->seg_k) return QSL_ERR_INVALID_ARG;
  const uint64_t d = cfg->d;
  const uint32_t L = cfg->num_segments;
  if (d == 0 || d >= (1ull << 32) || L == 0 || L > 16384) return QSL_ERR_INVALID_ARG;
  if (cfg->sparsifier > 1 || cfg->quantizer > 1) return QSL_ERR_INVALID_ARG;
  if (cfg->quantizer == QSL_QSGD && (cfg->s == 0 || cfg->s > 32768)) return QSL_ERR_INVALID_ARG;
  if (cfg->max_workers == 0 || cfg->max_workers > 1024) return QSL_ERR_INVALID_ARG;
  if (cfg->seg_offset[0] != 0 || cfg->seg_offset[L] != d) return QSL_ERR_INVALID_ARG;
  uint64_t K64 = 0;
  for (uint32_t l = 0; l < L; ++l) {
    if (cfg->seg_offset[l + 1] <= cfg->seg_offset[l]) return QSL_ERR_INVALID_ARG;
    const uint64_t size = cfg->seg_offset[l + 1] - cfg->seg_offset[l];
    if (cfg->seg_k[l] == 0 || cfg->seg_k[l] > size) return QSL_ERR_INVALID_ARG;
    K64 += cfg->seg_k[l];
  }
  if (K64 >= (1ull << 32)) return QSL_ERR_INVALID_ARG;

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
  ctx->timing = 0; ctx->ev_used = 0; ctx->ev_ms = 0; ctx->ev_launches = 0;
  ctx->slab = nullptr; ctx->h_status = nullptr;

  const uint32_t K = static_cast<uint32_t>(K64);
  const uint32_t s = cfg->quantizer == QSL_QSGD ? cfg->s : 1;
  const uint32_t w_idx = std::max(1u, bit_width_u64(d - 1));
  const uint32_t w_lev = cfg->quantizer == QSL_QSGD ? bit_width_u64(static_cast<uint64_t>(s) - 1) : 0;
  const uint32_t w_val = w_lev + 1;
  const bool counts = cfg->quantizer == QSL_QSGD && L > 1;
  uint64_t bits = 32 + 32ull * L + (counts ? 32ull * L : 0);
  bits += align_up(static_cast<uint64_t>(K) * w_idx, 32) + align_up(static_cast<uint64_t>(K) * w_val, 32);
  ctx->capacity = static_cast<size_t>(align_up(bits, 64) / 8);

  // per-segment plan: single-pass guessing ("fast") where the unit is large and sparse enough
  std::vector<SegInfo>& segs = ctx->segs;
  segs.resize(L);
  std::vector<TileInfo> tiles;
  std::vector<NormTile> ntiles;
  std::vector<uint32_t> fast;
  uint64_t pool_entries = 0;
  uint32_t koff = 0;
  bool has_general = false;
  for (uint32_t l = 0; l < L; ++l) {
    SegInfo& sg = segs[l];
    memset(&sg, 0, sizeof sg);
    sg.start = ctx->off[l]; sg.size = ctx->off[l + 1] - ctx->off[l];
    sg.k = ctx->k[l]; sg.koff = koff; koff += sg.k;
    sg.tile_base = static_cast<uint32_t>(tiles.size());
    const uint64_t nchunks = (sg.size + CHUNK - 1) / CHUNK;
    sg.ntiles = static_cast<uint32_t>((nchunks + CHUNKS_PER_TILE - 1) / CHUNKS_PER_TILE);
    for (uint32_t t = 0; t < sg.ntiles; ++t) {
      TileInfo ti; ti.seg = l; ti.first_chunk = t * CHUNKS_PER_TILE;
      ti.nchunks = static_cast<uint32_t>(std::min<uint64_t>(CHUNKS_PER_TILE, nchunks - ti.first_chunk)); ti.pad = 0;
      tiles.push_back(ti);
    }
    for (uint32_t f = 0; f < sg.k; f += NORM_TILE) {
      NormTile nt; nt.seg = l; nt.first = f; nt.count = std::min(NORM_TILE, sg.k - f); nt.pad = 0;
      ntiles.push_back(nt);
    }
    sg.mode = PATH_GENERAL;
    sg.T_static = 0xFFFFFFFFu;
    const double n = static_cast<double>(sg.size), p = static_cast<double>(sg.k) / n;
    if (!(cfg->flags & QSL_FLAG_NO_FAST_PATH) && sg.size >= (1u << 18)) {
      if (cfg->sparsifier == QSL_TOPK && static_cast<uint64_t>(sg.k) * 64 <= sg.size) {
        // candidates ~ alpha k; the sample must hold enough of them for the guess to sit below the
        // true threshold with ~6.5 sigma: (alpha - 1) sqrt(n_s p) >= 6.5 sqrt(alpha)
        const double alphas[4] = {1.5, 2.0, 3.0, 4.0};
        for (double alpha : alphas) {
          const double n_s = 42.25 * alpha / ((alpha - 1) * (alpha - 1) * p);
          if (n_s > n / 16) continue;
          sg.n_runs = static_cast<uint32_t>(std::ceil(n_s / 64.0));
          sg.r_s = static_cast<uint32_t>(std::ceil(alpha * (sg.n_runs * 64.0) * p));
          sg.pool_cap = static_cast<uint32_t>(std::min<double>(n, 4.0 * alpha * sg.k + 8192.0));
          sg.mode = PATH_FAST;
          break;
        }
      } else if (cfg->sparsifier == QSL_RANDK && static_cast<uint64_t>(sg.k) * 16 <= sg.size) {
        // the keys are uniform 32-bit words: keep those above the (1 - q) quantile, q = p + 7 sigma
        const double q = p + 7.0 * std::sqrt(p * (1 - p) / n);
        if (q < 0.25) {
          sg.T_static = static_cast<uint32_t>(std::floor(4294967296.0 * (1.0 - q)));
          sg.pool_cap = static_cast<uint32_t>(std::min<double>(n, q * n + 8.0 * std::sqrt(q * n) + 1024.0));
          sg.mode = PATH_FAST;
        }
      }
    }
    if (sg.mode == PATH_FAST) { fast.push_back(l); sg.pool_off = pool_entries; pool_entries += sg.pool_cap; }
    else has_general = true;
  }
  const uint32_t NT = static_cast<uint32_t>(tiles.size()), NNT = static_cast<uint32_t>(ntiles.size());
  const uint32_t QB = (K + QBLOCK - 1) / QBLOCK;
  const uint64_t R = ctx->Rmax, U = R * L;

  // one slab, carved
  uint64_t bytes = 0;
  auto carve = [&](uint64_t n) { const uint64_t o = bytes; bytes = align_up(bytes + n, 256); return o; };
  const uint64_t o_segs = carve(sizeof(SegInfo) * L), o_tiles = carve(sizeof(TileInfo) * NT);
  const uint64_t o_nt = carve(sizeof(NormTile) * std::max(1u, NNT)), o_fast = carve(4ull * std::max<size_t>(1, fast.size()));
  const uint64_t o_units = carve(sizeof(UnitState) * U);
  const uint64_t o_pool = carve(8ull * std::max<uint64_t>(1, pool_entries) * R);
  const uint64_t o_rec = carve(8ull * NT * R), o_cnt = carve(8ull * NT * R);
  const uint64_t o_hist = carve(4ull * HBINS * U), o_acc = carve(8ull * ACC_SLOTS * U);
  const uint64_t o_si = carve(4ull * K * R), o_sv = carve(4ull * K * R), o_sc = carve(4ull * K * R);
  const uint64_t o_blk = carve(4ull * QB * R), o_nnz = carve(4ull * R);
  const uint64_t o_vi = carve(4ull * K * R), o_vc = carve(4ull * K * R);
  const uint64_t o_status = carve(8), o_tmp = carve(4ull * 1024);
  if (hipMalloc(&ctx->slab, bytes) != hipSuccess) { delete ctx; return QSL_ERR_DEVICE; }
  char* base = static_cast<char*>(ctx->slab);
  bool ok = hipMemset(base + o_status, 0, 8) == hipSuccess;
  ok = ok && hipMemcpy(base + o_segs, segs.data(), sizeof(SegInfo) * L, hipMemcpyHostToDevice) == hipSuccess;
  ok = ok && hipMemcpy(base + o_tiles, tiles.data(), sizeof(TileInfo) * NT, hipMemcpyHostToDevice) == hipSuccess;
  if (NNT) ok = ok && hipMemcpy(base + o_nt, ntiles.data(), sizeof(NormTile) * NNT, hipMemcpyHostToDevice) == hipSuccess;
  if (!fast.empty()) ok = ok && hipMemcpy(base + o_fast, fast.data(), 4 * fast.size(), hipMemcpyHostToDevice) == hipSuccess;
  ok = ok && hipHostMalloc(reinterpret_cast<void**>(&ctx->h_status), 64, hipHostMallocDefault) == hipSuccess;
  if (!ok) { hipFree(ctx->slab); delete ctx; return QSL_ERR_DEVICE; }

  DevCtx& c = ctx->dc;
  c.segs = reinterpret_cast<const SegInfo*>(base + o_segs);
  c.tiles = reinterpret_cast<const TileInfo*>(base + o_tiles);
  c.ntiles = reinterpret_cast<const NormTile*>(base + o_nt);
  c.fast_segs = reinterpret_cast<const uint32_t*>(base + o_fast);
  c.units = reinterpret_cast<UnitState*>(base + o_units);
  c.pool = reinterpret_cast<uint2*>(base + o_pool); c.pool_stride = std::max<uint64_t>(1, pool_entries);
  c.tile_rec = reinterpret_cast<uint2*>(base + o_rec); c.tile_cnt = reinterpret_cast<uint2*>(base + o_cnt);
  c.hist = reinterpret_cast<uint32_t*>(base + o_hist); c.norm_acc = reinterpret_cast<uint64_t*>(base + o_acc);
  c.sel_idx = reinterpret_cast<uint32_t*>(base + o_si); c.sel_val = reinterpret_cast<uint32_t*>(base + o_sv);
  c.sel_code = reinterpret_cast<uint32_t*>(base + o_sc);
  c.blk_cnt = reinterpret_cast<uint32_t*>(base + o_blk); c.nnz_total = reinterpret_cast<uint32_t*>(base + o_nnz);
  c.surv_idx = reinterpret_cast<uint32_t*>(base + o_vi); c.surv_code = reinterpret_cast<uint32_t*>(base + o_vc);
  c.status = reinterpret_cast<uint32_t*>(base + o_status); c.any_fallback = c.status + 1;
  ctx->d_nnz_tmp = reinterpret_cast<uint32_t*>(base + o_tmp);
  c.d = d; c.seed = cfg->seed; c.L = L; c.K = K; c.NT = NT; c.NNT = NNT; c.QB = QB;
  c.nfast = static_cast<uint32_t>(fast.size()); c.s = s; c.w_idx = w_idx; c.w_lev = w_lev; c.w_val = w_val;
  c.sparsifier = cfg->sparsifier; c.quantizer = cfg->quantizer; c.has_general = has_general ? 1 : 0;
  c.cap_words = static_cast<uint32_t>(ctx->capacity / 4);
  *out = ctx;
  return QSL_OK;
}

extern "C" qsl_status qsl_destroy(qsl_ctx* ctx) {
  if (!ctx) return QSL_ERR_INVALID_ARG;
  hipStreamSynchronize(ctx->stream);
  for (hipEvent_t e : ctx->ev) hipEventDestroy(e);
  if (ctx->slab) hipFree(ctx->slab);
  if (ctx->h_status) hipHostFree(ctx->h_status);
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
static qsl_status launch_compress(qsl_ctx* ctx, const float* m, const float* delta, float* m_out, uint32_t worker0,
                                  uint32_t R, uint64_t round, uint8_t* msg, uint64_t* msg_bits, uint32_t* sel_idx,
                                  uint16_t* sel_level) {
  const DevCtx& c = ctx->dc;
  hipStream_t st = ctx->stream;
  const uint32_t U = R * c.L;
  k_init<<<dim3(static_cast<uint32_t>(std::min<uint64_t>(1024, (static_cast<uint64_t>(U) * HBINS + 255) / 256))), 256, 0, st>>>(c, R);
  if (SPARS == QSL_TOPK && c.nfast) {
    k_sample<<<dim3(SAMPLE_BLOCKS, c.nfast, R), BLOCK, 0, st>>>(c, m, delta);
    k_sample_scan<<<dim3(c.nfast, R), 1024, 0, st>>>(c);
  }
  const bool timed = ctx->timing != 0;
  if (timed) {
    if (ctx->ev_used + 2 > ctx->ev.size()) {
      for (int i = 0; i < 2; ++i) { hipEvent_t e; QSL_HIP(hipEventCreate(&e)); ctx->ev.push_back(e); }
    }
    QSL_HIP(hipEventRecord(ctx->ev[ctx->ev_used], st));
  }
  k_stream<SPARS><<<dim3(c.NT, R), BLOCK, 0, st>>>(c, m, delta, m_out, worker0, round);
  if (timed) { QSL_HIP(hipEventRecord(ctx->ev[ctx->ev_used + 1], st)); ctx->ev_used += 2; }

  const dim3 ugrid(c.L, R);
  const dim3 vgrid(std::min<uint32_t>(c.NT, 1024), R);
  if (c.nfast) {
    k_validate<<<dim3((U + 255) / 256), 256, 0, st>>>(c, U);
    k_pool_hist<0, SPARS><<<dim3(POOL_HIST_BLOCKS, c.nfast, R), BLOCK, 0, st>>>(c, worker0, round);
  }
  k_v_hist<0, SPARS><<<vgrid, BLOCK, 0, st>>>(c, m_out, worker0, round);
  k_hist_scan<0><<<ugrid, 1024, 0, st>>>(c);
  if (c.nfast) k_pool_hist<1, SPARS><<<dim3(POOL_HIST_BLOCKS, c.nfast, R), BLOCK, 0, st>>>(c, worker0, round);
  k_v_hist<1, SPARS><<<vgrid, BLOCK, 0, st>>>(c, m_out, worker0, round);
  k_hist_scan<1><<<ugrid, 1024, 0, st>>>(c);
  if (c.nfast) k_pool_hist<2, SPARS><<<dim3(POOL_HIST_BLOCKS, c.nfast, R), BLOCK, 0, st>>>(c, worker0, round);
  k_v_hist<2, SPARS><<<vgrid, BLOCK, 0, st>>>(c, m_out, worker0, round);
  k_hist_scan<2><<<ugrid, 1024, 0, st>>>(c);

  k_tile_count<SPARS><<<dim3(c.NT, R), BLOCK, 0, st>>>(c, m_out, worker0, round);
  k_tile_scan<<<ugrid, 1024, 0, st>>>(c);
  k_tile_write<SPARS><<<dim3(c.NT, R), BLOCK, 0, st>>>(c, m_out, worker0, round);

  k_norm<<<dim3(c.NNT, R), BLOCK, 0, st>>>(c);
  k_norm_finalize<<<dim3((U + 63) / 64), 64, 0, st>>>(c, U);
  k_quantize<<<dim3(c.QB, R), QBLOCK, 0, st>>>(c, m_out, worker0, round, sel_idx, sel_level);
  k_surv_scan<<<dim3(R), 1024, 0, st>>>(c);
  k_surv_compact<<<dim3(c.QB, R), QBLOCK, 0, st>>>(c);
  k_pack<<<dim3((c.cap_words + BLOCK - 1) / BLOCK, R), BLOCK, 0, st>>>(c, msg, msg_bits);
  QSL_HIP(hipGetLastError());
  return QSL_OK;
}

extern "C" qsl_status qsl_compress(qsl_ctx* ctx, const float* m, const float* delta, float* m_out, uint32_t worker0,
                                   uint32_t R, uint64_t round, uint8_t* msg, uint64_t* msg_bits, uint32_t* sel_idx,
                                   uint16_t* sel_level) {
  if (!ctx || !m || !delta || !m_out || !msg || R == 0 || R > ctx->Rmax || (round >> 62)) return QSL_ERR_INVALID_ARG;
  if (static_cast<uint64_t>(worker0) + R > (1ull << 32)) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(delta) | reinterpret_cast<uintptr_t>(m_out) |
       reinterpret_cast<uintptr_t>(sel_idx)) & 3) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(msg) | reinterpret_cast<uintptr_t>(msg_bits)) & 7) return QSL_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(sel_level) & 1) return QSL_ERR_INVALID_ARG;
  ctx->last_R = R;
  if (ctx->cfg.sparsifier == QSL_TOPK)
    return launch_compress<QSL_TOPK>(ctx, m, delta, m_out, worker0, R, round, msg, msg_bits, sel_idx, sel_level);
  return launch_compress<QSL_RANDK>(ctx, m, delta, m_out, worker0, R, round, msg, msg_bits, sel_idx, sel_level);
}

extern "C" qsl_status qsl_error_update(qsl_ctx* ctx, float* m, const float* delta, const uint8_t* msg, uint32_t R) {
  if (!ctx || !m || !delta || !msg || R == 0 || R > ctx->Rmax) return QSL_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(delta)) & 3) return QSL_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(msg) & 7) return QSL_ERR_INVALID_ARG;
  const DevCtx& c = ctx->dc;
  const uint64_t n = static_cast<uint64_t>(R) * c.d;
  const uint32_t blocks = static_cast<uint32_t>(std::min<uint64_t>((n + BLOCK * 4 - 1) / (BLOCK * 4), 1u << 16));
  k_add_rows<<<dim3(blocks), BLOCK, 0, ctx->stream>>>(m, delta, n);
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
  k_aggregate<<<dim3((c.K + BLOCK - 1) / BLOCK, R), BLOCK, 0, ctx->stream>>>(c, msg, rows, R, scale, accumulate, out);
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
  const bool counts = c.quantizer == QSL_QSGD && c.L > 1;
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
    o[0] = us[u].path; o[1] = us[u].cand; o[2] = us[u].tau; o[3] = us[u].n_gt; o[4] = us[u].need; o[5] = us[u].T;
    o[6] = us[u].scale_bits; o[7] = us[u].nnz;
  }
  *n_units = U;
  return QSL_OK;
}

extern "C" qsl_status qsl_timing_enable(qsl_ctx* ctx, int enabled) {
  if (!ctx) return QSL_ERR_INVALID_ARG;
  ctx->timing = enabled; ctx->ev_used = 0; ctx->ev_ms = 0; ctx->ev_launches = 0;
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
