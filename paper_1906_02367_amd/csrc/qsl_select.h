// qsl_select.h -- Exact selection of the k largest rank keys of every unit (Section 2.2) and their ordered compaction:
// k_select<0..2> (radix digits over the whole vector), k_full (k = size), k_tile_count and k_tile_write (ordered
// output, exact norm digits); the slot rows of the guessing units.
// Part of the single translation unit qsl.hip (included there, in this order: device, layout, select,
// encode, stream, lean, dense, decode); not a public header.
#pragma once

#include "qsl_device.h"
#include "qsl_layout.h"

namespace {

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

// The 16 bytes of a slot row that this lane reads (and, for Rand_k, the 8 bytes of its key line), as loaded: kept
// in this form while several rows are in flight, parsed when the row's turn comes (a parsed row takes twice the
// registers).  Rows past the end, and lanes past the unit's last chunk, read as empty.
struct RawRow { uint4 q; uint2 kq; };

__device__ __forceinline__ RawRow load_slot_row(const uint2* slots, const uint32_t* slot_key, uint32_t lpc, uint32_t nwt,
                                                uint64_t row, uint64_t nrows) {
  RawRow r;
  const uint32_t lane = lane_id();
  r.q = make_uint4(0, 0, 0, 0);
  r.kq = make_uint2(0, 0);
  if (row < nrows && ((row * 64 + lane) >> (__ffs(lpc) - 1)) < nwt) {                                                 // lpc: 4, 8, 16 or 32
    r.q = reinterpret_cast<const uint4*>(slots)[row * 64 + lane];
    if (slot_key) r.kq = reinterpret_cast<const uint2*>(slot_key)[row * 64 + lane];
  }
  return r;
}

__device__ __forceinline__ SlotRow parse_slot_row(const RawRow& raw, uint32_t lpc) {
  SlotRow r;
  const uint32_t lane = lane_id();
  const uint32_t sub = lane & (lpc - 1);
  const uint4 q = raw.q;
  r.key0 = raw.kq.x; r.key1 = raw.kq.y;
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

constexpr int ROWS_IN_FLIGHT = 8;                 // slot rows a wave of the guessing units' kernels loads at a time

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

// Digit LEVEL of the k-th largest key of a unit on the multi-pass path: the blocks of the unit read v and build the
// digit's histogram (LDS, then a few global atomics per bin); which bin the previous digit fell in is recomputed by
// every block from the previous kernel's histogram.  A guessing unit is listed here too, for the call in which its
// guess failed and the host asked for this chain (`safe` launches); otherwise its blocks return at once.
template <int LEVEL, int SPARS>
__global__ __launch_bounds__(BIG) void k_select(DevCtx c, SegInfo one, const float* v, uint32_t worker0, uint64_t round,
                                                uint32_t R) {
  __shared__ uint32_t lh[HBINS];
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[6];
  // a single-segment context carries its plan in the kernel arguments: one dependent load less per block
  // one-dimensional grid, the workers innermost: the blocks of the plan's list start in list order (heaviest
  // first) for all workers alike, instead of worker after worker
  const uint32_t li = blockIdx.x / R, w = blockIdx.x % R;
  SelInfo si; si.seg = 0; si.j = li;
  if (c.L != 1) si = c.sels[li];
  const SegInfo sg = c.L == 1 ? one : c.segs[si.seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + si.seg;
  UnitState* usp = &c.units[u];
  const UnitState us = *usp;
  if (us.path == PATH_FAST && !us.fell_back) return;         // its guess held: k_lean_* select it
  uint32_t* hist = c.hist + u * 3 * HBINS;
  for (uint32_t i = threadIdx.x; i < HBINS; i += BIG) lh[i] = 0;
  __syncthreads();
  uint32_t prefix = 0, k_rem = sg.k;
  if (LEVEL == 0) {
    if (us.path != PATH_FAST && threadIdx.x == 0 && si.j == 0) { usp->cand = 0; usp->fell_back = 0; usp->nnz = 0; }
  } else {
    uint32_t above;
    if (LEVEL == 1) {
      // (for a guessing unit whose guess failed also rank r_warm >= k: its next guess comes from this histogram of
      // the whole unit, as after a fresh sample)
      find2_from_top<BIG>(hist, sg.k, us.path == PATH_FAST ? sg.r_warm : sg.k, scratch, result, false);
      const uint32_t bin = result[0];
      above = result[1];
      prefix = bin << 20; k_rem = sg.k - above;
      if (SPARS == QSL_TOPK && us.path == PATH_FAST && threadIdx.x == 0 && si.j == 0) {
        uint32_t sh = 11;
        while (sh < 20 && (1u << (sh - 11)) < bin + 1 - result[2]) ++sh;
        usp->T_next = result[2] << 20; usp->sh_next = sh;
      }
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
  {
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
// A "compaction block" covers a contiguous range of groups of 16 chunks of v (a group at a time: each wave
// 4 chunks, a lane 16 coordinates of a chunk; one group per block while the unit has at most 256 groups).
// k_tile_count leaves the number of selected coordinates of every block; k_tile_write sums the earlier
// blocks' numbers to know where it writes.  A guessing unit whose guess failed runs here with the blocks
// the plan gives it for that case.
//
// Exact norms: every |v| (or v^2) is an integer multiple of 2^-149 (2^-298); its 32-bit digits are
// added into 64-bit counters; integer addition commutes, so any schedule gives the same sum.
// ------------------------------------------------------------------------------------------------
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
// M^power (power = 1 .. 4, M < 2^24) as hi * 2^64 + lo
__device__ __forceinline__ void power_of_mantissa(uint32_t M, uint32_t power, uint64_t* lo, uint64_t* hi) {
  const uint64_t sq = static_cast<uint64_t>(M) * M;         // < 2^48
  *hi = 0;
  if (power == 1) *lo = M;
  else if (power == 2) *lo = sq;
  else if (power == 3) { *lo = sq * M; *hi = __umul64hi(sq, M); }
  else { *lo = sq * sq; *hi = __umul64hi(sq, sq); }
}
// |v|^power = M^power * 2^(power (e1 - 150)): its 32-bit digits above 2^(-149 power) into the row
__device__ __forceinline__ void add_digits(uint64_t* mine, uint32_t bits, uint32_t power) {
  const uint32_t ab = bits & 0x7FFFFFFFu;
  const uint32_t ex = ab >> 23, frac = ab & 0x7FFFFFu;
  const uint32_t M = ex ? (frac | 0x800000u) : frac;       // |v| = M * 2^(max(ex,1) - 150)
  const uint32_t e1 = ex ? ex : 1u;
  if (M == 0) return;
  if (power == 2) {
    const uint64_t sq = static_cast<uint64_t>(M) * M;       // < 2^48;  v^2 = sq * 2^(2 e1 - 300)
    const uint32_t p = 2u * e1 - 2u;                        // bit position above 2^-298
    const uint32_t q = p >> 5, r = p & 31u;
    const uint64_t lo = sq << r;                            // low 64 bits of sq * 2^r  (r <= 30)
    const uint64_t hi = r ? (sq >> (64 - r)) : 0;
    lds_add(&mine[q], lo & 0xFFFFFFFFu); lds_add(&mine[q + 1], lo >> 32);
    if (hi) lds_add(&mine[q + 2], hi);
  } else if (power == 1) {
    const uint32_t p = e1 - 1u;                             // bit position above 2^-149
    const uint32_t q = p >> 5, r = p & 31u;
    const uint64_t sh = static_cast<uint64_t>(M) << r;      // < 2^55
    lds_add(&mine[q], sh & 0xFFFFFFFFu);
    if (sh >> 32) lds_add(&mine[q + 1], sh >> 32);
  } else {                                                  // cubes and fourth powers: up to 96 bits, four digits
    uint64_t lo, hi;
    power_of_mantissa(M, power, &lo, &hi);
    const uint32_t p = power * (e1 - 1u), q = p >> 5, r = p & 31u;
    const uint64_t a0 = lo << r;
    const uint64_t a1 = (hi << r) | (r ? lo >> (64 - r) : 0);
    lds_add(&mine[q], a0 & 0xFFFFFFFFu); lds_add(&mine[q + 1], a0 >> 32);
    if (a1) { lds_add(&mine[q + 2], a1 & 0xFFFFFFFFu); if (a1 >> 32) lds_add(&mine[q + 3], a1 >> 32); }
  }
}

// the general-path groups [g_lo, g_hi) of one unit, by one 256-thread block.
// WRITE = false: returns (in *tot_gt, *tot_eq, valid in thread 0) how many coordinates of these groups have key > tau / == tau.
// WRITE = true: writes the selected ones, in coordinate order, starting at ranks (gt0, eq0).
template <int SPARS, bool WRITE>
__device__ void general_groups(const SegInfo& sg, const float* vp, const RandKey& rk, Thresh th,
                               uint32_t g_lo, uint32_t g_hi, uint32_t gt0, uint32_t eq0, uint32_t* oi, uint32_t* ov,
                               uint64_t* mine, uint32_t power, uint32_t* s_cnt /*[2][GGROUP + 1]*/,
                               uint32_t* tot_gt, uint32_t* tot_eq) {
  constexpr uint32_t STAGE = 512;                  // list entries per wave (WRITE only)
  __shared__ uint32_t stage_pos[WRITE ? (BLOCK / 64) * STAGE : 1];
  __shared__ uint2 stage_iv[WRITE ? (BLOCK / 64) * STAGE : 1];
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
      // The selected coordinates are few per lane (a dense k is still a few per cent), so a loop that stores and
      // adds digits where it finds one runs its body once per element position with one or two lanes active.
      // The lanes park what they find in a list of the wave instead (rank, coordinate, value); the list is
      // then worked off 64 entries at a time by all lanes.
      uint32_t staged = 0;                                            // entries in the wave's list (wave-uniform)
      auto flush = [&]() {
        // the list is private to the wave, whose lanes run in lockstep: order the LDS traffic only
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (uint32_t o = 0; o < staged; o += 64) {
          if (o + lane < staged) {
            const uint32_t pos = stage_pos[wave * STAGE + o + lane];
            const uint2 e = stage_iv[wave * STAGE + o + lane];
            oi[pos] = e.x; ov[pos] = e.y;
            add_digits(mine, e.y, power);
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");      // ... and before the list is refilled
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        staged = 0;
      };
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
          if (staged + 256 > STAGE) flush();                         // room for the 4 x 64 elements of this step
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const bool is_gt = (gn >> j) & 1u, is_eq = (qn >> j) & 1u;
            const bool take = is_gt || (is_eq && my_eq < th.need);
            const uint64_t tb = __ballot(take);
            if (take) {
              const uint32_t slot = wave * STAGE + staged + popc_below(tb);
              stage_pos[slot] = my_gt + min(my_eq, th.need);
              stage_iv[slot] = make_uint2(static_cast<uint32_t>(sg.start + cb + t * 256 + lane * 4 + j),
                                          __float_as_uint(val[q][t][j]));
            }
            staged += static_cast<uint32_t>(__popcll(tb));
            my_gt += is_gt; my_eq += is_eq;
          }
          base_gt += tg; base_eq += tq;
        }
      }
      flush();
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
// units with k = size: every coordinate is selected, so there is nothing to search (the error-feedback
// schemes without sparsification that Section 5 compares with, as this operator).  The blocks of a unit
// copy contiguous ranges of 4096-coordinate tiles of v into the selected arrays -- position = coordinate --
// and add the digits of the norm.
// ------------------------------------------------------------------------------------------------
typedef uint32_t u4u __attribute__((ext_vector_type(4), aligned(4)));

__global__ __launch_bounds__(BLOCK) void k_full(DevCtx c, const float* v) {
  __shared__ uint64_t acc[ACC_ROWS * (ACC_SLOTS + 1)];
  const SelInfo si = c.fulls[blockIdx.x];
  const uint32_t w = blockIdx.y;
  const SegInfo sg = c.segs[si.seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + si.seg;
  const float* vp = v + static_cast<uint64_t>(w) * c.d + sg.start;
  uint32_t* oi = c.sel_idx + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint32_t* ov = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff;
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t power = norm_power(c.quantizer);
  uint64_t* mine = acc + (wave * 8 + (lane & 7u)) * acc_stride(c.quantizer);
  for (uint32_t i = threadIdx.x; i < ACC_ROWS * acc_stride(c.quantizer); i += BLOCK) acc[i] = 0;
  __syncthreads();
  const uint64_t ntiles = (sg.size + 4095) / 4096;
  const uint32_t nb = static_cast<uint32_t>(ntiles < MAX_FULL_BLOCKS ? ntiles : MAX_FULL_BLOCKS);
  const uint64_t t_lo = ntiles * si.j / nb, t_hi = ntiles * (si.j + 1) / nb;
  for (uint64_t tile = t_lo; tile < t_hi; ++tile) {
    f4u x[4];
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {                       // a wave instruction covers 1 KiB of the row
      const uint64_t e = tile * 4096 + q * 1024 + threadIdx.x * 4;
      x[q] = f4u{0.f, 0.f, 0.f, 0.f};
      if (e + 4 <= sg.size) x[q] = *reinterpret_cast<const f4u*>(vp + e);
      else {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) if (e + j < sg.size) x[q][j] = vp[e + j];
      }
    }
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      const uint64_t e = tile * 4096 + q * 1024 + threadIdx.x * 4;
      const uint32_t i0 = static_cast<uint32_t>(sg.start + e);
      u4u bits, idx;
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) { bits[j] = __float_as_uint(x[q][j]); idx[j] = i0 + j; }
      if (e + 4 <= sg.size) {
        *reinterpret_cast<u4u*>(oi + e) = idx;
        *reinterpret_cast<u4u*>(ov + e) = bits;
      } else {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) if (e + j < sg.size) { oi[e + j] = idx[j]; ov[e + j] = bits[j]; }
      }
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) if (e + j < sg.size) add_digits(mine, bits[j], power);
    }
  }
  __syncthreads();
  uint64_t* ga = c.norm_acc + u * ACC_SLOTS;
  for (uint32_t s = wave; s < acc_slots(c.quantizer); s += BLOCK / 64) {
    uint64_t x = lane < ACC_ROWS ? acc[lane * acc_stride(c.quantizer) + s] : 0;
    x = wave_sum64(x);
    if (lane == 0 && x) atomicAdd(reinterpret_cast<unsigned long long*>(ga + s), static_cast<unsigned long long>(x));
  }
  if (threadIdx.x == 0 && si.j == 0) {
    UnitState* us = &c.units[u];
    us->cand = 0; us->fell_back = 0; us->tau = 0; us->need = 0; us->n_gt = sg.k; us->nnz = 0;
  }
}

template <int SPARS>
__global__ __launch_bounds__(BLOCK) void k_tile_count(DevCtx c, SegInfo one, const float* v, uint32_t worker0, uint64_t round,
                                                      uint32_t R) {
  __shared__ uint32_t s_cnt[2 * GGROUP + 2], result[2];
  __shared__ uint64_t scratch[17];
  const uint32_t li = blockIdx.x / R, w = blockIdx.x % R;             // workers innermost, as in k_select
  CbInfo cb; cb.seg = 0; cb.b = li;
  if (c.L != 1) cb = c.cbs[li];
  const SegInfo sg = c.L == 1 ? one : c.segs[cb.seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + cb.seg;
  const UnitState us = c.units[u];
  if (us.path == PATH_FAST && !us.fell_back) return;         // its guess held: k_lean_* select it
  const Thresh th = last_digit(c, u, us, scratch, result);
  if (threadIdx.x == 0 && cb.b == 0) { c.units[u].tau = th.tau; c.units[u].need = th.need; c.units[u].n_gt = sg.k - th.need; }
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  uint2* out = c.cb_cnt + static_cast<uint64_t>(w) * c.NCB + sg.cb_base + cb.b;
  uint32_t g_lo, g_hi;
  fallback_range(sg, cb.b, &g_lo, &g_hi);
  uint32_t tg = 0, tq = 0;
  general_groups<SPARS, false>(sg, v + static_cast<uint64_t>(w) * c.d + sg.start, rk, th, g_lo, g_hi, 0, 0, nullptr,
                               nullptr, nullptr, false, s_cnt, &tg, &tq);
  if (threadIdx.x == 0) *out = make_uint2(tg, tq);
}

template <int SPARS>
__global__ __launch_bounds__(BLOCK) void k_tile_write(DevCtx c, SegInfo one, const float* v, uint32_t worker0, uint64_t round,
                                                      uint32_t R) {
  __shared__ uint64_t acc[ACC_ROWS * (ACC_SLOTS + 1)];      // a row per 8 lanes of a wave: short atomic queues
  __shared__ uint32_t s_cnt[2 * GGROUP + 2];
  __shared__ uint64_t scratch[17], s_part[4];
  const uint32_t li = blockIdx.x / R, w = blockIdx.x % R;             // workers innermost, as in k_select
  CbInfo cb; cb.seg = 0; cb.b = li;
  if (c.L != 1) cb = c.cbs[li];
  const SegInfo sg = c.L == 1 ? one : c.segs[cb.seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + cb.seg;
  const UnitState us = c.units[u];
  if (us.path == PATH_FAST && !us.fell_back) return;         // its guess held: k_lean_* select it
  Thresh th; th.tau = us.tau; th.need = us.need;
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t power = norm_power(c.quantizer);
  uint64_t* mine = acc + (wave * 8 + (lane & 7u)) * acc_stride(c.quantizer);
  for (uint32_t i = threadIdx.x; i < ACC_ROWS * acc_stride(c.quantizer); i += BLOCK) acc[i] = 0;   // published by the barrier below
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
  {
    uint32_t g_lo, g_hi;
    fallback_range(sg, cb.b, &g_lo, &g_hi);
    uint32_t tg, tq;
    general_groups<SPARS, true>(sg, v + static_cast<uint64_t>(w) * c.d + sg.start, rk, th, g_lo, g_hi, gt0, eq0, oi, ov,
                                mine, power, s_cnt, &tg, &tq);
  }
  __syncthreads();
  uint64_t* ga = c.norm_acc + u * ACC_SLOTS;
  for (uint32_t s = wave; s < acc_slots(c.quantizer); s += 4) {
    uint64_t x = lane < ACC_ROWS ? acc[lane * acc_stride(c.quantizer) + s] : 0;
    x = wave_sum64(x);
    if (lane == 0 && x) atomicAdd(reinterpret_cast<unsigned long long*>(ga + s), static_cast<unsigned long long>(x));
  }
}

}  // namespace
