// qsl_lean.h -- The guessing units' way from the candidates in the chunk slots to encoded entries, in three launches:
//   k_lean_hist   histogram of the candidates' keys in 4096 bins of 2^sh keys above the guess T; candidates per wave
//   k_lean_mark   the bin of the k-th largest candidate ("threshold bin"); the candidates, in coordinate order, into
//                 the unit's dense list; per wave the number that lie in higher bins -- all of them selected, so the
//                 exact digits of their norm are added up here; the few candidates inside the threshold bin go to a
//                 short list; the guess and the bin width of the next call
//   k_lean_emit   every block ranks the short list (exact threshold, ties to the lower coordinate), finishes the
//                 norm and the fp32 scale, and its waves write their selected candidates in order: coordinate, code
//                 (Definition 1, example 1 / Definition 2), error update on the transmitted ones (Algorithm 1, second
//                 worker line).  Extra blocks, one per guessing unit, take the units whose guess failed or whose
//                 threshold bin is too crowded for the list: one block selects exactly, by radix digits, from the
//                 dense list or from v itself.
//   k_lean_one    the three steps above in one launch, for a unit that has a single block in them
// The result never depends on the guess or on the bins: they only decide how much work the exact selection is.
// Part of the single translation unit qsl.hip (included after qsl_encode.h); not a public header.
#pragma once

#include "qsl_device.h"
#include "qsl_layout.h"
#include "qsl_select.h"
#include "qsl_encode.h"

namespace {

constexpr uint32_t LEAN_ROWS = 64;         // accumulator rows of a 1024-thread block (8 lanes of a wave share one)

struct LeanUnit {
  SegInfo sg; uint32_t seg, j, w; uint64_t u;
  const uint2* slots; const uint2* ovf; const uint32_t* slot_key; const uint32_t* ovf_key;
  uint2* d0; uint32_t* d0k; uint32_t* wcnt; uint32_t* wsel;
  uint32_t nrows, gw, rpw; uint64_t r_lo, r_hi;
};

template <int SPARS>
__device__ __forceinline__ void lean_unit(const DevCtx& c, const SegInfo& one, uint32_t R, LeanUnit& lu) {
  const uint32_t li = blockIdx.x / R;
  lu.w = blockIdx.x % R;                        // workers innermost: the heaviest blocks of every worker start first
  SelInfo si; si.seg = 0; si.j = li;
  if (c.L != 1) si = c.fsels[li];
  lu.seg = si.seg; lu.j = si.j;
  lu.sg = c.L == 1 ? one : c.segs[si.seg];
  const SegInfo& sg = lu.sg;
  lu.u = static_cast<uint64_t>(lu.w) * c.L + si.seg;
  lu.slots = c.slots + static_cast<uint64_t>(lu.w) * c.slot_stride + sg.slot_off;
  lu.ovf = c.ovf + static_cast<uint64_t>(lu.w) * c.ovf_stride + sg.ovf_off;
  lu.slot_key = SPARS == QSL_RANDK ? c.slot_key + static_cast<uint64_t>(lu.w) * c.slot_stride + sg.slot_off : nullptr;
  lu.ovf_key = SPARS == QSL_RANDK ? c.ovf_key + static_cast<uint64_t>(lu.w) * c.ovf_stride + sg.ovf_off : nullptr;
  lu.d0 = c.d0 + static_cast<uint64_t>(lu.w) * c.d0_stride + sg.d0_off;
  lu.d0k = c.d0_key + static_cast<uint64_t>(lu.w) * c.d0_stride + sg.d0_off;
  lu.wcnt = c.wave_cnt + static_cast<uint64_t>(lu.w) * c.NWC + sg.wc_base;
  lu.wsel = c.wave_sel + static_cast<uint64_t>(lu.w) * c.NWC + sg.wc_base;
  lu.nrows = static_cast<uint32_t>((static_cast<uint64_t>(sg.nwt) * sg.lpc + 63) >> 6);   // < 2^20
  const uint32_t nwaves = sg.nsel * (BIG / 64);
  lu.gw = si.j * (BIG / 64) + (threadIdx.x >> 6);
  lu.rpw = (lu.nrows + nwaves - 1) / nwaves;     // every wave a contiguous range of slot rows
  lu.r_lo = static_cast<uint64_t>(lu.gw) * lu.rpw;
  lu.r_hi = lu.r_lo + lu.rpw < lu.nrows ? lu.r_lo + lu.rpw : lu.nrows;
}

// sum of cnt[g] over the waves g < gw of the unit (at most MAX_SELECT_BLOCKS * 16 = 1024 waves: 16 loads in flight)
__device__ __forceinline__ uint32_t waves_before(const uint32_t* cnt, uint32_t gw) {
  const uint32_t lane = lane_id();
  uint32_t part[MAX_SELECT_BLOCKS * (BIG / 64) / WAVE];
#pragma unroll
  for (uint32_t i = 0; i < MAX_SELECT_BLOCKS * (BIG / 64) / WAVE; ++i) {
    const uint32_t g = i * WAVE + lane;
    part[i] = g < gw ? cnt[g] : 0u;
  }
  uint32_t x = 0;
#pragma unroll
  for (uint32_t i = 0; i < MAX_SELECT_BLOCKS * (BIG / 64) / WAVE; ++i) x += part[i];
  return wave_sum(x);
}

// ------------------------------------------------------------------------------------------------
// first launch: the candidates' histogram
// ------------------------------------------------------------------------------------------------
template <int SPARS>
__global__ __launch_bounds__(BIG) void k_lean_hist(DevCtx c, SegInfo one, uint32_t R) {
  __shared__ uint32_t lh[HBINS];
  __shared__ uint32_t s_ctr[CTR_LINES];
  LeanUnit lu;
  lean_unit<SPARS>(c, one, R, lu);
  const SegInfo& sg = lu.sg;
  UnitState* usp = &c.units[lu.u];
  const uint32_t T = usp->T, sh = usp->sh;
  RawRow rr[ROWS_IN_FLIGHT];                     // independent accesses in flight; rows past the end read as empty
#pragma unroll
  for (int b = 0; b < ROWS_IN_FLIGHT; ++b) rr[b] = load_slot_row(lu.slots, lu.slot_key, sg.lpc, sg.nwt, lu.r_lo + b, lu.r_hi);   // issued before anything waits
  for (uint32_t i = threadIdx.x; i < HBINS; i += BIG) lh[i] = 0;
  if (threadIdx.x < CTR_LINES) s_ctr[threadIdx.x] = c.ctr[(lu.u * CTR_LINES + threadIdx.x) * PAD];
  __syncthreads();
  // a guess that produced too few candidates, or more than there is room for, is discarded here
  uint32_t cand = 0;
  for (uint32_t i = 0; i < NSUB; ++i) cand += s_ctr[i];
  const bool failed = s_ctr[CTR_FAIL] != 0 || cand < sg.k || cand > sg.d0_cap;
  if (threadIdx.x == 0 && lu.j == 0) {
    usp->cand = cand; usp->fell_back = failed; usp->nnz = 0;
    if (failed && SPARS == QSL_TOPK) {
      // no histogram to place the next guess with: move it by a quarter of a binade (a whole one when even half of k
      // is missing) towards where the candidates are
      const uint32_t step = cand < sg.k / 2 ? 1u << 24 : 1u << 22;
      usp->T_next = cand < sg.k ? (T > step ? T - step : 0u) : (T < 0xFFFFFFFFu - step ? T + step : T);
      usp->sh_next = sh;
    }
  }
  if (failed) return;
  const uint32_t lane = lane_id();
  uint32_t seen = 0;
  for (uint64_t row0 = lu.r_lo; row0 < lu.r_hi; row0 += ROWS_IN_FLIGHT) {
    if (row0 != lu.r_lo) {
#pragma unroll
      for (int b = 0; b < ROWS_IN_FLIGHT; ++b) rr[b] = load_slot_row(lu.slots, lu.slot_key, sg.lpc, sg.nwt, row0 + b, lu.r_hi);
    }
#pragma unroll
    for (int b = 0; b < ROWS_IN_FLIGHT; ++b) {
      if (row0 + b >= lu.r_hi) break;                              // uniform over the wave
      const SlotRow r = parse_slot_row(rr[b], sg.lpc);
      seen += r.n;
      if (!r.spill) {
        if (r.has0) atomicAdd(&lh[lean_bin(SPARS == QSL_TOPK ? key_of_value(r.bits0) : r.key0, T, sh)], 1u);
        if (r.has1) atomicAdd(&lh[lean_bin(SPARS == QSL_TOPK ? key_of_value(r.bits1) : r.key1, T, sh)], 1u);
      }
      // chunks whose candidates went to the overflow pool: the whole wave reads each one's entries, 64 at a time
      for (uint64_t spilled = __ballot(r.spill); spilled; spilled &= spilled - 1) {
        const int holder = __ffsll(static_cast<unsigned long long>(spilled)) - 1;
        const uint32_t cnt = __shfl(r.count, holder, WAVE), at = __shfl(r.ovf_at, holder, WAVE);
        for (uint32_t e = lane; e < cnt; e += WAVE) {
          const uint32_t key = SPARS == QSL_TOPK ? key_of_value(lu.ovf[at + e].y) : lu.ovf_key[at + e];
          atomicAdd(&lh[lean_bin(key, T, sh)], 1u);
        }
      }
    }
  }
  seen = wave_sum(seen);
  if (lane == 0) lu.wcnt[lu.gw] = seen;
  __syncthreads();
  flush_hist(lh, c.hist + lu.u * 3 * HBINS);
}

// ------------------------------------------------------------------------------------------------
// second launch: threshold bin, dense list, what is certainly selected, the short list
// ------------------------------------------------------------------------------------------------
template <int SPARS>
__global__ __launch_bounds__(BIG) void k_lean_mark(DevCtx c, SegInfo one, uint32_t R) {
  __shared__ uint64_t acc[LEAN_ROWS * (ACC_SLOTS + 1)];
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[6];
  LeanUnit lu;
  lean_unit<SPARS>(c, one, R, lu);
  const SegInfo& sg = lu.sg;
  UnitState* usp = &c.units[lu.u];
  const UnitState us = *usp;
  if (us.fell_back) return;
  const uint32_t T = us.T, sh = us.sh;
  // the loads that depend on nothing are issued first: this wave's first slot rows, the earlier waves' counts
  RawRow rr[ROWS_IN_FLIGHT];
#pragma unroll
  for (int b = 0; b < ROWS_IN_FLIGHT; ++b) rr[b] = load_slot_row(lu.slots, lu.slot_key, sg.lpc, sg.nwt, lu.r_lo + b, lu.r_hi);
  uint32_t off = waves_before(lu.wcnt, lu.gw);      // where this wave's candidates go in the dense list
  for (uint32_t i = threadIdx.x; i < LEAN_ROWS * acc_stride(c.quantizer); i += BIG) acc[i] = 0;     // published by the scan's barriers
  // rank k: the threshold's bin; rank r_warm >= k: where the next call's guess goes
  find2_from_top<BIG>(c.hist + lu.u * 3 * HBINS, sg.k, sg.r_warm, scratch, result, false);
  const uint32_t taubin = result[0], above = result[1], in_bin = result[4];
  const bool crowded = in_bin > LISTCAP;
  if (threadIdx.x == 0 && lu.j == 0) {
    usp->taubin = taubin; usp->above = above; usp->crowded = crowded;
    if (SPARS == QSL_TOPK) {
      // Next call: the lower edge of the bin of rank r_warm, if this call has that many candidates; if it has fewer
      // the guess was tighter than planned and moves down by as much as the threshold lies above it.  Bins: 4096
      // over four times the distance from the new guess to this call's threshold.
      const uint32_t tau_lo = T + (taubin << sh);                     // lower edge of the threshold's bin (no overflow: a candidate's key lies there)
      uint32_t T_next;
      if (result[5] >= sg.r_warm) T_next = T + (result[2] << sh);
      else { const uint32_t down = max(tau_lo - T, 1u << sh); T_next = T > down ? T - down : 0u; }
      const uint32_t span = max(tau_lo - T_next, 1u) >> 10;           // bin width so that the threshold lands near bin 1024
      uint32_t sh_next = 0;
      while (sh_next < 20 && (1u << sh_next) < span) ++sh_next;
      if (taubin == HBINS - 1) sh_next = min(20u, max(sh_next, sh + 4));   // the threshold lies beyond the bins: much wider ones
      usp->T_next = T_next; usp->sh_next = sh_next;
    }
  }
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t power = norm_power(c.quantizer);
  uint64_t* mine = acc + ((wave & 7u) * 8 + (lane & 7u)) * acc_stride(c.quantizer);
  uint32_t* cursor = c.ctr + (lu.u * CTR_LINES + CTR_LIST) * PAD;
  uint4* list = c.tlist + (static_cast<uint64_t>(lu.w) * c.nfast + sg.fidx) * LISTCAP;
  uint32_t n_above = 0;
  // one candidate per lane (or none): into the dense list; counted and added to the norm if it lies above the
  // threshold's bin; appended to the short list if it lies inside.  Called by all lanes of the wave together.
  auto visit = [&](bool has, uint32_t p, uint32_t idx, uint32_t bits, uint32_t key) {
    bool inside = false;
    if (has) {
      lu.d0[p] = make_uint2(idx, bits);
      if (SPARS == QSL_RANDK) lu.d0k[p] = key;
      const uint32_t b = lean_bin(key, T, sh);
      if (b > taubin) { ++n_above; add_digits(mine, bits, power); }
      else inside = b == taubin && !crowded;
    }
    const uint64_t ib = __ballot(inside);
    if (ib != 0) {                                   // wave-uniform
      const int first = __ffsll(static_cast<unsigned long long>(ib)) - 1;
      uint32_t base = 0;
      if (static_cast<int>(lane) == first) base = atomicAdd(cursor, static_cast<uint32_t>(__popcll(ib)));
      base = __shfl(base, first, WAVE);
      const uint32_t q = base + popc_below(ib);
      if (inside && q < LISTCAP) list[q] = make_uint4(p, bits, key, idx);
    }
  };
  for (uint64_t row0 = lu.r_lo; row0 < lu.r_hi; row0 += ROWS_IN_FLIGHT) {
    if (row0 != lu.r_lo) {
#pragma unroll
      for (int b = 0; b < ROWS_IN_FLIGHT; ++b) rr[b] = load_slot_row(lu.slots, lu.slot_key, sg.lpc, sg.nwt, row0 + b, lu.r_hi);
    }
#pragma unroll
    for (int b = 0; b < ROWS_IN_FLIGHT; ++b) {
      if (row0 + b >= lu.r_hi) break;                              // uniform over the wave
      const SlotRow r = parse_slot_row(rr[b], sg.lpc);
      uint32_t tot;
      const uint32_t pos = off + wave_exclusive_scan32(r.n, &tot);
      off += tot;
      const bool h0 = !r.spill && r.has0, h1 = !r.spill && r.has1;
      if (__ballot(h0 || h1) != 0) {
        visit(h0, pos, r.idx0, r.bits0, SPARS == QSL_TOPK ? key_of_value(r.bits0) : r.key0);
        visit(h1, pos + (h0 ? 1u : 0u), r.idx1, r.bits1, SPARS == QSL_TOPK ? key_of_value(r.bits1) : r.key1);
      }
      for (uint64_t spilled = __ballot(r.spill); spilled; spilled &= spilled - 1) {
        const int holder = __ffsll(static_cast<unsigned long long>(spilled)) - 1;
        const uint32_t cnt = __shfl(r.count, holder, WAVE), at = __shfl(r.ovf_at, holder, WAVE);
        const uint32_t first = __shfl(pos, holder, WAVE);
        for (uint32_t e0 = 0; e0 < cnt; e0 += WAVE) {                // all lanes stay in the loop: visit is collective
          const uint32_t e = e0 + lane;
          uint2 ent = make_uint2(0, 0); uint32_t key = 0;
          if (e < cnt) { ent = lu.ovf[at + e]; key = SPARS == QSL_TOPK ? key_of_value(ent.y) : lu.ovf_key[at + e]; }
          visit(e < cnt, first + e, ent.x, ent.y, key);
        }
      }
    }
  }
  n_above = wave_sum(n_above);
  if (lane == 0) lu.wsel[lu.gw] = n_above;
  __syncthreads();
  uint64_t* ga = c.norm_acc + lu.u * ACC_SLOTS;
  for (uint32_t s = wave; s < acc_slots(c.quantizer); s += BIG / 64) {
    const uint64_t x = wave_sum64(acc[lane * acc_stride(c.quantizer) + s]);       // LEAN_ROWS = 64 rows: one per lane
    if (lane == 0 && x) atomicAdd(reinterpret_cast<unsigned long long*>(ga + s), static_cast<unsigned long long>(x));
  }
}

// ------------------------------------------------------------------------------------------------
// A unit of at most 40,960 coordinates that is too dense for guessing, whole, by one block of 1024 threads: a wave
// takes up to 2560 consecutive coordinates, read again from v (which the cache holds) for each of the three radix
// digits and for the ordered pass; one block-wide scan and ballots inside the waves order the output.  Selection, norm, codes and error update
// without a launch in between.
// ------------------------------------------------------------------------------------------------
template <int SPARS>
__device__ void block_unit(const DevCtx& c, const SegInfo& sg, uint32_t w, uint64_t u, const float* vp, uint32_t worker0,
                           uint64_t round, float* m_out, uint32_t* dbg_idx, uint16_t* dbg_level, uint32_t* lh,
                           uint64_t* acc, uint64_t* scratch, uint32_t* result, float* s_scale, uint32_t* s_count) {
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t n = static_cast<uint32_t>(sg.size);                 // <= BLOCK_MAX
  // Wave wv takes the coordinates [wv * gw * 256, (wv + 1) * gw * 256) of the unit, in gw <= 10 groups of 256: lane l holds
  // the four coordinates (g * 64 + l) * 4 .. + 3 of group g, so that a load of the wave is 1 KB in a row.  (A thread with
  // 36 consecutive coordinates of its own made every load touch 64 cache lines, and the first pass over a unit of 36,864
  // coordinates, which comes from memory, took 14 of the block's 43 us.)
  // A pass: the loads of five groups are issued together, then f(e, bits[4], keys[4], nv) sees the lane's four
  // coordinates of each group (the first nv of them lie inside the unit), group after group; every lane of the wave
  // makes the same calls.
  const uint32_t gw = (n + (BIG / 64) * 256 - 1) / ((BIG / 64) * 256);
  const uint32_t wbase = wave * gw * 256;
  auto pass = [&](auto&& f) {
    constexpr uint32_t G = 5;                        // (ten at once: the compiler spills, 600 bytes per lane)
    for (uint32_t g0 = 0; g0 < gw; g0 += G) {
      f4u x[G];
#pragma unroll
      for (uint32_t g = 0; g < G; ++g) {
        const uint32_t e = wbase + (g0 + g) * 256 + lane * 4;
        x[g] = f4u{0.f, 0.f, 0.f, 0.f};
        if (g0 + g < gw) {
          if (e + 4 <= n) x[g] = *reinterpret_cast<const f4u*>(vp + e);
          else {
#pragma unroll
            for (uint32_t j = 0; j < 4; ++j) if (e + j < n) x[g][j] = vp[e + j];
          }
        }
      }
#pragma unroll
      for (uint32_t g = 0; g < G; ++g) {
        if (g0 + g >= gw) continue;                                  // uniform over the wave
        const uint32_t e = wbase + (g0 + g) * 256 + lane * 4;
        const uint32_t nv = e < n ? min(4u, n - e) : 0u;
        Words4 rw = {{0u, 0u, 0u, 0u}};
        if (SPARS == QSL_RANDK && nv) rw = rand_words4(rk, static_cast<uint32_t>(sg.start) + e);
        uint32_t bits[4], keys[4];
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
          bits[j] = __float_as_uint(x[g][j]);
          keys[j] = SPARS == QSL_TOPK ? key_of_value(bits[j]) : rw.w[j];
        }
        f(e, bits, keys, nv);
      }
    }
  };
  for (uint32_t i = threadIdx.x; i < HBINS; i += BIG) lh[i] = 0;
  for (uint32_t i = threadIdx.x; i < LEAN_ROWS * acc_stride(c.quantizer); i += BIG) acc[i] = 0;
  __syncthreads();
  uint32_t above, bin;
  // the three digits of the k-th largest key
  pass([&](uint32_t, const uint32_t*, const uint32_t* keys, uint32_t nv) {
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) if (j < nv) atomicAdd(&lh[keys[j] >> 20], 1u);
  });
  __syncthreads();
  bin = find_from_top<BIG>(lh, sg.k, &above, scratch, result, true);
  uint32_t prefix = bin << 20, k_rem = sg.k - above;
  pass([&](uint32_t, const uint32_t*, const uint32_t* keys, uint32_t nv) {
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) if (j < nv && (keys[j] >> 20) == (prefix >> 20)) atomicAdd(&lh[(keys[j] >> 8) & 0xFFFu], 1u);
  });
  __syncthreads();
  bin = find_from_top<BIG>(lh, k_rem, &above, scratch, result, true);
  prefix |= bin << 8; k_rem -= above;
  pass([&](uint32_t, const uint32_t*, const uint32_t* keys, uint32_t nv) {
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) if (j < nv && (keys[j] >> 8) == (prefix >> 8)) atomicAdd(&lh[keys[j] & 0xFFu], 1u);
  });
  __syncthreads();
  bin = find_from_top<BIG, 1024>(lh, k_rem, &above, scratch, result, true);      // bins 256 .. 1023 are empty
  const uint32_t tau = prefix | bin, need = k_rem - above;
  // ordered compaction: key > tau, and the first `need` coordinates with key == tau
  uint32_t n_gt = 0, n_eq = 0;
  pass([&](uint32_t, const uint32_t*, const uint32_t* keys, uint32_t nv) {
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) if (j < nv) { n_gt += keys[j] > tau; n_eq += keys[j] == tau; }
  });
  uint64_t total;
  const uint64_t ex = block_exclusive_scan64((static_cast<uint64_t>(n_eq) << 32) | n_gt, scratch, &total);
  // the wave's coordinates follow those of the waves before it: what these hold is what lane 0's prefix says
  const uint64_t ex0 = __shfl(ex, 0, WAVE);
  uint32_t run_gt = static_cast<uint32_t>(ex0), run_eq = static_cast<uint32_t>(ex0 >> 32);
  uint32_t* oi = c.sel_idx + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint32_t* ov = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint64_t* mine = acc + ((wave & 7u) * 8 + (lane & 7u)) * acc_stride(c.quantizer);
  const uint32_t power = norm_power(c.quantizer);
  if (__ballot(n_gt != 0 || n_eq != 0) != 0) {
    pass([&](uint32_t e, const uint32_t* bits, const uint32_t* keys, uint32_t nv) {
      // inside a group the coordinates run lane after lane: what the lower lanes hold comes first
      uint32_t bg = 0, bq = 0, tg = 0, tq = 0;
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) {
        const uint64_t b1 = __ballot(j < nv && keys[j] > tau), b2 = __ballot(j < nv && keys[j] == tau);
        bg += popc_below(b1); tg += static_cast<uint32_t>(__popcll(b1));
        bq += popc_below(b2); tq += static_cast<uint32_t>(__popcll(b2));
      }
      uint32_t my_gt = run_gt + bg, my_eq = run_eq + bq;
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) {
        const bool is_gt = j < nv && keys[j] > tau, is_eq = j < nv && keys[j] == tau;
        if (is_gt || (is_eq && my_eq < need)) {
          const uint32_t pos = my_gt + min(my_eq, need);
          if (pos < sg.k) { oi[pos] = static_cast<uint32_t>(sg.start) + e + j; ov[pos] = bits[j]; add_digits(mine, bits[j], power); }
        }
        my_gt += is_gt; my_eq += is_eq;
      }
      run_gt += tg; run_eq += tq;
    });
  }
  if (threadIdx.x == 0) { c.units[u].cand = 0; c.units[u].fell_back = 0; }
  block_encode_tail<BIG, LEAN_ROWS>(c, sg, w, u, tau, need, worker0, round, m_out, dbg_idx, dbg_level, acc, s_scale, s_count);
}

template <int SPARS>
__global__ __launch_bounds__(BIG) void k_block_units(DevCtx c, uint32_t R, float* m_out, uint32_t worker0, uint64_t round,
                                                     uint32_t* dbg_idx, uint16_t* dbg_level) {
  __shared__ uint32_t lh[HBINS];
  __shared__ uint64_t acc[LEAN_ROWS * (ACC_SLOTS + 1)];
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[2], s_count;
  __shared__ float s_scale;
  const uint32_t seg = c.small_segs[blockIdx.x / R], w = blockIdx.x % R;       // workers innermost, largest units first
  const SegInfo sg = c.segs[seg];
  block_unit<SPARS>(c, sg, w, static_cast<uint64_t>(w) * c.L + seg, m_out + static_cast<uint64_t>(w) * c.d + sg.start,
                    worker0, round, m_out, dbg_idx, dbg_level, lh, acc, scratch, result, &s_scale, &s_count);
}

// ------------------------------------------------------------------------------------------------
// exact selection of one unit by one block of 1024 threads, by radix digits (12 + 12 + 8 bits) and an ordered pass,
// followed by the norm and the encoding of the k selected coordinates: for a unit whose guess failed (FROM_V: the
// keys come from v itself) or whose threshold bin was too crowded for the short list (from the dense list).  Slow
// for a large unit read from v, and rare: the host switches to the multi-pass kernels when it has happened.
// ------------------------------------------------------------------------------------------------
template <int SPARS, bool FROM_V>
__device__ void block_select_encode(const DevCtx& c, const SegInfo& sg, uint32_t w, uint64_t u, const float* vp,
                                    const uint2* d0, const uint32_t* d0k, uint64_t n, uint32_t worker0, uint64_t round,
                                    float* m_out, uint32_t* dbg_idx, uint16_t* dbg_level, uint32_t* lh, uint64_t* acc,
                                    uint64_t* scratch, uint32_t* result, float* s_scale, uint32_t* s_count) {
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  auto load = [&](uint64_t i, uint32_t* idx, uint32_t* bits, uint32_t* key) {
    if (FROM_V) {
      *idx = static_cast<uint32_t>(sg.start + i);
      *bits = __float_as_uint(vp[i]);
      *key = SPARS == QSL_TOPK ? key_of_value(*bits) : rand_word(rk, *idx);
    } else {
      const uint2 e = d0[i];
      *idx = e.x; *bits = e.y;
      *key = SPARS == QSL_TOPK ? key_of_value(e.y) : d0k[i];
    }
  };
  for (uint32_t i = threadIdx.x; i < HBINS; i += BIG) lh[i] = 0;
  for (uint32_t i = threadIdx.x; i < LEAN_ROWS * acc_stride(c.quantizer); i += BIG) acc[i] = 0;
  __syncthreads();
  uint32_t prefix = 0, k_rem = sg.k, above, idx, bits, key;
  for (uint64_t i = threadIdx.x; i < n; i += BIG) { load(i, &idx, &bits, &key); atomicAdd(&lh[key >> 20], 1u); }
  __syncthreads();
  uint32_t bin_w = 0;
  if (FROM_V && SPARS == QSL_TOPK) bin_w = find_from_top<BIG>(lh, sg.r_warm, &above, scratch, result, false);
  uint32_t bin = find_from_top<BIG>(lh, k_rem, &above, scratch, result, true);
  if (FROM_V && SPARS == QSL_TOPK && threadIdx.x == 0) {
    // the guess had failed: the next one comes from this histogram of the whole unit, as after a fresh sample
    uint32_t sh = 11;
    while (sh < 20 && (1u << (sh - 11)) < bin + 1 - bin_w) ++sh;
    c.units[u].T_next = bin_w << 20; c.units[u].sh_next = sh;
  }
  prefix = bin << 20; k_rem -= above;
  for (uint64_t i = threadIdx.x; i < n; i += BIG) {
    load(i, &idx, &bits, &key);
    if ((key >> 20) == (prefix >> 20)) atomicAdd(&lh[(key >> 8) & 0xFFFu], 1u);
  }
  __syncthreads();
  bin = find_from_top<BIG>(lh, k_rem, &above, scratch, result, true);
  prefix |= bin << 8; k_rem -= above;
  for (uint64_t i = threadIdx.x; i < n; i += BIG) {
    load(i, &idx, &bits, &key);
    if ((key >> 8) == (prefix >> 8)) atomicAdd(&lh[key & 0xFFu], 1u);
  }
  __syncthreads();
  bin = find_from_top<BIG, 1024>(lh, k_rem, &above, scratch, result, true);      // bins 256 .. 1023 are empty
  const uint32_t tau = prefix | bin, need = k_rem - above;
  // ordered pass: key > tau, and the first `need` with key == tau; a thread takes 4 consecutive entries of a tile
  uint32_t* oi = c.sel_idx + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint32_t* ov = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff;
  const uint32_t power = norm_power(c.quantizer);
  uint64_t* mine = acc + ((wave & 7u) * 8 + (lane & 7u)) * acc_stride(c.quantizer);
  uint32_t run_gt = 0, run_eq = 0;
  for (uint64_t base = 0; base < n; base += 4ull * BIG) {
    uint32_t ix[4], bt[4], gm = 0, qm = 0;
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      const uint64_t i = base + threadIdx.x * 4ull + q;
      ix[q] = 0; bt[q] = 0;
      if (i < n) {
        load(i, &ix[q], &bt[q], &key);
        gm |= (key > tau ? 1u : 0u) << q; qm |= (key == tau ? 1u : 0u) << q;
      }
    }
    uint64_t total;
    const uint64_t ex = block_exclusive_scan64((static_cast<uint64_t>(__popc(qm)) << 32) | __popc(gm), scratch, &total);
    uint32_t my_gt = run_gt + static_cast<uint32_t>(ex), my_eq = run_eq + static_cast<uint32_t>(ex >> 32);
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      const bool is_gt = (gm >> q) & 1u, is_eq = (qm >> q) & 1u;
      if (is_gt || (is_eq && my_eq < need)) {
        const uint32_t pos = my_gt + min(my_eq, need);
        if (pos < sg.k) { oi[pos] = ix[q]; ov[pos] = bt[q]; add_digits(mine, bt[q], power); }
      }
      my_gt += is_gt; my_eq += is_eq;
    }
    run_gt += static_cast<uint32_t>(total); run_eq += static_cast<uint32_t>(total >> 32);
  }
  block_encode_tail<BIG, LEAN_ROWS>(c, sg, w, u, tau, need, worker0, round, m_out, dbg_idx, dbg_level, acc, s_scale, s_count);
}

// ------------------------------------------------------------------------------------------------
// third launch: exact threshold from the short list, ordered output, codes, error update
// ------------------------------------------------------------------------------------------------
template <int SPARS>
__global__ __launch_bounds__(BIG) void k_lean_emit(DevCtx c, SegInfo one, uint32_t R, uint32_t n_regular, float* m_out,
                                                   uint32_t worker0, uint64_t round, uint32_t* dbg_idx,
                                                   uint16_t* dbg_level, int safe) {
  __shared__ uint32_t lh[HBINS];                                  // the block-wide selection's histogram
  __shared__ uint64_t acc[LEAN_ROWS * (ACC_SLOTS + 1)];
  __shared__ uint4 s_list[LISTCAP];
  __shared__ uint8_t s_sel[LISTCAP];
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[2], s_tau, s_need, s_count;
  __shared__ float s_scale;
  if (blockIdx.x >= n_regular) {
    // one block per guessing unit, idle unless the unit could not go the short way
    const uint32_t bi = blockIdx.x - n_regular;
    const uint32_t seg = c.L == 1 ? 0u : c.fast_segs[bi / R], w = bi % R;
    const SegInfo sg = c.L == 1 ? one : c.segs[seg];
    const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
    if (c.none != 0 && sg.nsel == 1) return;                      // k_lean_one looks after its units itself
    const UnitState us = c.units[u];
    if (us.fell_back) {
      if (safe) return;                                           // the multi-pass kernels of this call took the unit
      if (threadIdx.x == 0) *c.host_flag = 1u;                    // the host will ask for them on its next calls
      block_select_encode<SPARS, true>(c, sg, w, u, m_out + static_cast<uint64_t>(w) * c.d + sg.start, nullptr, nullptr,
                                       sg.size, worker0, round, m_out, dbg_idx, dbg_level, lh, acc, scratch, result, &s_scale,
                                       &s_count);
    } else if (us.crowded) {
      block_select_encode<SPARS, false>(c, sg, w, u, nullptr, c.d0 + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off,
                                        c.d0_key + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off, us.cand, worker0,
                                        round, m_out, dbg_idx, dbg_level, lh, acc, scratch, result, &s_scale, &s_count);
    }
    return;
  }
  LeanUnit lu;
  lean_unit<SPARS>(c, one, R, lu);
  const SegInfo& sg = lu.sg;
  // the candidates' histogram has served (k_lean_mark was its last reader): this block's share of it back to zero
  for (uint32_t i = lu.j * BIG + threadIdx.x; i < HBINS; i += sg.nsel * BIG) c.hist[lu.u * 3 * HBINS + i] = 0;
  UnitState* usp = &c.units[lu.u];
  const UnitState us = *usp;
  if (us.fell_back || us.crowded) return;
  const uint32_t T = us.T, sh = us.sh, taubin = us.taubin;
  const uint32_t k_rem = sg.k - us.above;                         // how many of the threshold bin's candidates are selected (>= 1)
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t power = norm_power(c.quantizer);
  // The loads that depend on nothing are issued together: the list's length and entries (a thread per entry of the
  // whole array; what lies beyond the length is stale and ignored), the digits of the norm, the counts of the waves.
  static_assert(LISTCAP <= BIG, "a thread per list entry");
  const uint4* glist = c.tlist + (static_cast<uint64_t>(lu.w) * c.nfast + sg.fidx) * LISTCAP;
  const uint32_t n_list = min(c.ctr[(lu.u * CTR_LINES + CTR_LIST) * PAD], LISTCAP);
  uint4 me = make_uint4(0, 0, 0, 0);
  if (threadIdx.x < LISTCAP) me = glist[threadIdx.x];
  const uint64_t my_digit = threadIdx.x < acc_slots(c.quantizer) ? c.norm_acc[lu.u * ACC_SLOTS + threadIdx.x] : 0;
  const uint32_t cnt = lu.wcnt[lu.gw];
  const uint32_t d_off = waves_before(lu.wcnt, lu.gw);
  uint32_t s_off = waves_before(lu.wsel, lu.gw);
  // ... and, once the wave knows where its candidates are, the first 64 of them
  uint2 ent_first = make_uint2(0, 0);
  uint32_t key_first = 0;
  if (lane < cnt) { ent_first = lu.d0[d_off + lane]; if (SPARS == QSL_RANDK) key_first = lu.d0k[d_off + lane]; }
  // the short list, ranked by (key descending, place in the dense list ascending = coordinate ascending)
  if (threadIdx.x == 0) { s_need = 0; s_tau = 0; }
  for (uint32_t i = threadIdx.x; i < ACC_SLOTS + 1; i += BIG) acc[i] = 0;
  if (threadIdx.x < n_list) s_list[threadIdx.x] = me;
  __syncthreads();
  bool sel = false;
  if (threadIdx.x < n_list) {
    uint32_t rank = 0;
    for (uint32_t j = 0; j < n_list; ++j) {
      const uint4 o = s_list[j];
      rank += (o.z > me.z || (o.z == me.z && o.x < me.x)) ? 1u : 0u;
    }
    sel = rank < k_rem;
    s_sel[threadIdx.x] = sel;
    if (rank == k_rem - 1) s_tau = me.z;                          // the k-th largest key of the unit
    if (sel) add_digits(acc, me.y, power);                      // the rest of the norm (LDS atomics on one row)
  }
  __syncthreads();
  if (sel && me.z == s_tau) atomicAdd(&s_need, 1u);
  // the scale: the digits k_lean_mark added up, plus the selected entries of the list
  if (threadIdx.x < acc_slots(c.quantizer)) acc[threadIdx.x] += my_digit;
  __syncthreads();
  if (wave == 0) {
    const float sc = finalize_scale(acc, c.quantizer, sg.k);
    if (lane == 0) s_scale = sc;
  }
  __syncthreads();
  const UnitScale usc = unit_scale(c, s_scale, sg.k);
  if (threadIdx.x == 0 && lu.j == 0) {
    usp->tau = s_tau; usp->need = s_need; usp->n_gt = sg.k - s_need; usp->scale_bits = __float_as_uint(usc.sent);
  }
  // this wave's candidates: a contiguous range of the dense list; where its selected ones go
  {
    uint32_t x = 0;
    for (uint32_t j = lane; j < n_list; j += WAVE) x += (s_sel[j] && s_list[j].x < d_off) ? 1u : 0u;
    s_off += wave_sum(x);
  }
  const RandKey rk1 = make_rand_key(c.seed, worker0 + lu.w, round, 1);
  uint32_t nsent = 0;
  for (uint32_t e0 = 0; e0 < cnt; e0 += WAVE) {
    const uint32_t e = e0 + lane;
    const uint2 ent = ent_first;                                  // loaded one step ahead
    const uint32_t key = key_first;
    if (e + WAVE < cnt) { ent_first = lu.d0[d_off + e + WAVE]; if (SPARS == QSL_RANDK) key_first = lu.d0k[d_off + e + WAVE]; }
    uint32_t bin = 0;
    if (e < cnt) bin = lean_bin(SPARS == QSL_TOPK ? key_of_value(ent.y) : key, T, sh);
    bool take = e < cnt && bin > taubin;
    const bool maybe = e < cnt && bin == taubin;
    if (__ballot(maybe) != 0) {                                   // rare: look the entry up in the short list
      for (uint32_t j = 0; j < n_list; ++j) {
        const uint32_t p = s_list[j].x;
        if (maybe && p == d_off + e && s_sel[j]) take = true;
      }
    }
    const uint64_t tb = __ballot(take);
    const uint32_t pos = s_off + popc_below(tb);
    bool sent = false;
    if (take && pos < sg.k) {
      const uint64_t slot = static_cast<uint64_t>(lu.w) * c.K + sg.koff + pos;
      sent = encode_entry(c, lu.w, slot, ent.x, ent.y, usc, rk1, m_out, dbg_idx, dbg_level);
    }
    if (is_qsgd(c.quantizer)) {
      // survivors per block of 256 slots: the slots of one step are consecutive, so they touch at most two blocks
      const uint64_t sb = __ballot(sent);
      if (sb != 0) {
        const uint32_t b_first = (sg.koff + s_off) >> 8;
        const bool in_first = ((sg.koff + pos) >> 8) == b_first;
        const uint32_t n0 = static_cast<uint32_t>(__popcll(__ballot(sent && in_first)));
        const uint32_t n1 = static_cast<uint32_t>(__popcll(sb)) - n0;
        if (lane == 0) {
          uint32_t* bc = c.blk_cnt + static_cast<uint64_t>(lu.w) * c.QB;
          if (n0) atomicAdd(&bc[b_first], n0);
          if (n1) atomicAdd(&bc[b_first + 1], n1);
          nsent += n0 + n1;
        }
      }
    }
    s_off += static_cast<uint32_t>(__popcll(tb));
  }
  if (is_qsgd(c.quantizer) && c.L > 1 && lane == 0 && nsent) atomicAdd(&usp->nnz, nsent);
}

// ------------------------------------------------------------------------------------------------
// A guessing unit that the plan gives a single block in the three kernels above needs none of their launch
// boundaries: what they hand each other through memory (histogram, per-wave counts, norm digits, short list) one
// block can keep in LDS, with barriers where they had kernel ends.  Same steps, same results; the dense list is still
// written (the rescue of a crowded threshold bin reads it, and so does the ordered output).
// ------------------------------------------------------------------------------------------------
template <int SPARS>
__global__ __launch_bounds__(BIG) void k_lean_one(DevCtx c, SegInfo one, uint32_t R, float* m_out, uint32_t worker0,
                                                  uint64_t round, uint32_t* dbg_idx, uint16_t* dbg_level, int safe) {
  __shared__ uint32_t lh[HBINS];
  __shared__ uint64_t acc[LEAN_ROWS * (ACC_SLOTS + 1)];
  __shared__ uint4 s_list[LISTCAP];
  __shared__ uint8_t s_sel[LISTCAP];
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[6], s_ctr[CTR_LINES], s_wcnt[BIG / 64], s_wsel[BIG / 64], s_nlist, s_tau, s_need, s_count;
  __shared__ float s_scale;
  constexpr uint32_t NW = BIG / 64;
  const uint32_t w = blockIdx.x % R;                 // workers innermost, heaviest units first
  const uint32_t seg = c.L == 1 ? 0u : c.one_segs[blockIdx.x / R];
  const SegInfo sg = c.L == 1 ? one : c.segs[seg];
  const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
  UnitState* usp = &c.units[u];
  const UnitState us = *usp;
  const uint32_t T = us.T, sh = us.sh;
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint2* slots = c.slots + static_cast<uint64_t>(w) * c.slot_stride + sg.slot_off;
  const uint2* ovf = c.ovf + static_cast<uint64_t>(w) * c.ovf_stride + sg.ovf_off;
  const uint32_t* slot_key = SPARS == QSL_RANDK ? c.slot_key + static_cast<uint64_t>(w) * c.slot_stride + sg.slot_off : nullptr;
  const uint32_t* ovf_key = SPARS == QSL_RANDK ? c.ovf_key + static_cast<uint64_t>(w) * c.ovf_stride + sg.ovf_off : nullptr;
  uint2* d0 = c.d0 + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
  uint32_t* d0k = c.d0_key + static_cast<uint64_t>(w) * c.d0_stride + sg.d0_off;
  const uint32_t nrows = static_cast<uint32_t>((static_cast<uint64_t>(sg.nwt) * sg.lpc + 63) >> 6);
  const uint32_t rpw = (nrows + NW - 1) / NW;        // every wave a contiguous range of slot rows
  const uint64_t r_lo = static_cast<uint64_t>(wave) * rpw;
  const uint64_t r_hi = r_lo + rpw < nrows ? r_lo + rpw : nrows;
  const uint32_t power = norm_power(c.quantizer);
  const uint32_t st = acc_stride(c.quantizer);
  constexpr int RIF = SPARS == QSL_RANDK ? 4 : ROWS_IN_FLIGHT;   // rows in flight (a Rand_k row carries its keys: more registers)

  // ---- the candidates' histogram and the number each wave holds (what k_lean_hist does)
  RawRow rr[RIF];
#pragma unroll
  for (int b = 0; b < RIF; ++b) rr[b] = load_slot_row(slots, slot_key, sg.lpc, sg.nwt, r_lo + b, r_hi);
  for (uint32_t i = threadIdx.x; i < HBINS; i += BIG) lh[i] = 0;
  for (uint32_t i = threadIdx.x; i < LEAN_ROWS * st; i += BIG) acc[i] = 0;
  if (threadIdx.x < CTR_LINES) s_ctr[threadIdx.x] = c.ctr[(u * CTR_LINES + threadIdx.x) * PAD];
  if (threadIdx.x == 0) { s_nlist = 0; s_need = 0; s_tau = 0; s_count = 0; }
  __syncthreads();
  uint32_t cand = 0;
  for (uint32_t i = 0; i < NSUB; ++i) cand += s_ctr[i];
  const bool failed = s_ctr[CTR_FAIL] != 0 || cand < sg.k || cand > sg.d0_cap;
  if (threadIdx.x == 0) {
    usp->cand = cand; usp->fell_back = failed; usp->nnz = 0; usp->crowded = 0;
    if (failed && SPARS == QSL_TOPK) {                // as in k_lean_hist: towards where the candidates are
      const uint32_t step = cand < sg.k / 2 ? 1u << 24 : 1u << 22;
      usp->T_next = cand < sg.k ? (T > step ? T - step : 0u) : (T < 0xFFFFFFFFu - step ? T + step : T);
      usp->sh_next = sh;
    }
  }
  if (failed) {
    if (safe) return;                                 // the multi-pass kernels of this call take the unit
    if (threadIdx.x == 0) *c.host_flag = 1u;
    __syncthreads();
    block_select_encode<SPARS, true>(c, sg, w, u, m_out + static_cast<uint64_t>(w) * c.d + sg.start, nullptr, nullptr, sg.size,
                                     worker0, round, m_out, dbg_idx, dbg_level, lh, acc, scratch, result, &s_scale, &s_count);
    return;
  }
  uint32_t seen = 0;
  for (uint64_t row0 = r_lo; row0 < r_hi; row0 += RIF) {
    if (row0 != r_lo) {
#pragma unroll
      for (int b = 0; b < RIF; ++b) rr[b] = load_slot_row(slots, slot_key, sg.lpc, sg.nwt, row0 + b, r_hi);
    }
#pragma unroll
    for (int b = 0; b < RIF; ++b) {
      if (row0 + b >= r_hi) break;
      const SlotRow r = parse_slot_row(rr[b], sg.lpc);
      seen += r.n;
      if (!r.spill) {
        if (r.has0) atomicAdd(&lh[lean_bin(SPARS == QSL_TOPK ? key_of_value(r.bits0) : r.key0, T, sh)], 1u);
        if (r.has1) atomicAdd(&lh[lean_bin(SPARS == QSL_TOPK ? key_of_value(r.bits1) : r.key1, T, sh)], 1u);
      }
      for (uint64_t spilled = __ballot(r.spill); spilled; spilled &= spilled - 1) {
        const int holder = __ffsll(static_cast<unsigned long long>(spilled)) - 1;
        const uint32_t cnt = __shfl(r.count, holder, WAVE), at = __shfl(r.ovf_at, holder, WAVE);
        for (uint32_t e = lane; e < cnt; e += WAVE) {
          const uint32_t key = SPARS == QSL_TOPK ? key_of_value(ovf[at + e].y) : ovf_key[at + e];
          atomicAdd(&lh[lean_bin(key, T, sh)], 1u);
        }
      }
    }
  }
  seen = wave_sum(seen);
  if (lane == 0) s_wcnt[wave] = seen;
  // the first rows again, for the second walk (they come from the cache now)
#pragma unroll
  for (int b = 0; b < RIF; ++b) rr[b] = load_slot_row(slots, slot_key, sg.lpc, sg.nwt, r_lo + b, r_hi);
  __syncthreads();

  // ---- threshold bin, dense list, what is certainly selected, the short list (what k_lean_mark does)
  find2_from_top<BIG>(lh, sg.k, sg.r_warm, scratch, result, false);
  const uint32_t taubin = result[0], above = result[1], in_bin = result[4];
  const bool crowded = in_bin > LISTCAP;
  if (threadIdx.x == 0) {
    usp->taubin = taubin; usp->above = above; usp->crowded = crowded;
    if (SPARS == QSL_TOPK) {                          // the next call's guess and bin width, as in k_lean_mark
      const uint32_t tau_lo = T + (taubin << sh);
      uint32_t T_next;
      if (result[5] >= sg.r_warm) T_next = T + (result[2] << sh);
      else { const uint32_t down = max(tau_lo - T, 1u << sh); T_next = T > down ? T - down : 0u; }
      const uint32_t span = max(tau_lo - T_next, 1u) >> 10;
      uint32_t sh_next = 0;
      while (sh_next < 20 && (1u << sh_next) < span) ++sh_next;
      if (taubin == HBINS - 1) sh_next = min(20u, max(sh_next, sh + 4));
      usp->T_next = T_next; usp->sh_next = sh_next;
    }
  }
  uint32_t off = 0;
  for (uint32_t g = 0; g < wave; ++g) off += s_wcnt[g];
  const uint32_t d_off = off, cnt_w = s_wcnt[wave];
  uint64_t* mine = acc + ((wave & 7u) * 8 + (lane & 7u)) * st;
  uint32_t n_above = 0;
  auto visit = [&](bool has, uint32_t p, uint32_t idx, uint32_t bits, uint32_t key) {
    bool inside = false;
    if (has) {
      d0[p] = make_uint2(idx, bits);
      if (SPARS == QSL_RANDK) d0k[p] = key;
      const uint32_t b = lean_bin(key, T, sh);
      if (b > taubin) { ++n_above; add_digits(mine, bits, power); }
      else inside = b == taubin && !crowded;
    }
    const uint64_t ib = __ballot(inside);
    if (ib != 0) {                                   // wave-uniform
      const int first = __ffsll(static_cast<unsigned long long>(ib)) - 1;
      uint32_t base = 0;
      if (static_cast<int>(lane) == first) base = atomicAdd(&s_nlist, static_cast<uint32_t>(__popcll(ib)));
      base = __shfl(base, first, WAVE);
      const uint32_t q = base + popc_below(ib);
      if (inside && q < LISTCAP) s_list[q] = make_uint4(p, bits, key, idx);
    }
  };
  for (uint64_t row0 = r_lo; row0 < r_hi; row0 += RIF) {
    if (row0 != r_lo) {
#pragma unroll
      for (int b = 0; b < RIF; ++b) rr[b] = load_slot_row(slots, slot_key, sg.lpc, sg.nwt, row0 + b, r_hi);
    }
#pragma unroll
    for (int b = 0; b < RIF; ++b) {
      if (row0 + b >= r_hi) break;
      const SlotRow r = parse_slot_row(rr[b], sg.lpc);
      uint32_t tot;
      const uint32_t pos = off + wave_exclusive_scan32(r.n, &tot);
      off += tot;
      const bool h0 = !r.spill && r.has0, h1 = !r.spill && r.has1;
      if (__ballot(h0 || h1) != 0) {
        visit(h0, pos, r.idx0, r.bits0, SPARS == QSL_TOPK ? key_of_value(r.bits0) : r.key0);
        visit(h1, pos + (h0 ? 1u : 0u), r.idx1, r.bits1, SPARS == QSL_TOPK ? key_of_value(r.bits1) : r.key1);
      }
      for (uint64_t spilled = __ballot(r.spill); spilled; spilled &= spilled - 1) {
        const int holder = __ffsll(static_cast<unsigned long long>(spilled)) - 1;
        const uint32_t cnt = __shfl(r.count, holder, WAVE), at = __shfl(r.ovf_at, holder, WAVE);
        const uint32_t first = __shfl(pos, holder, WAVE);
        for (uint32_t e0 = 0; e0 < cnt; e0 += WAVE) {
          const uint32_t e = e0 + lane;
          uint2 ent = make_uint2(0, 0); uint32_t key = 0;
          if (e < cnt) { ent = ovf[at + e]; key = SPARS == QSL_TOPK ? key_of_value(ent.y) : ovf_key[at + e]; }
          visit(e < cnt, first + e, ent.x, ent.y, key);
        }
      }
    }
  }
  n_above = wave_sum(n_above);
  if (lane == 0) s_wsel[wave] = n_above;
  __threadfence_block();                             // the dense list is read back below, by other waves too
  __syncthreads();
  if (crowded) {                                     // more ties in the threshold's bin than the short list holds
    block_select_encode<SPARS, false>(c, sg, w, u, nullptr, d0, d0k, cand, worker0, round, m_out, dbg_idx, dbg_level, lh, acc,
                                      scratch, result, &s_scale, &s_count);
    return;
  }

  // ---- exact threshold from the short list, the scale, ordered output and codes (what k_lean_emit does)
  // this wave's first candidates, issued before the reductions
  uint2 ent_first = make_uint2(0, 0);
  uint32_t key_first = 0;
  if (lane < cnt_w) { ent_first = d0[d_off + lane]; if (SPARS == QSL_RANDK) key_first = d0k[d_off + lane]; }
  {                                                  // the accumulator rows added up into row 0 (as block_encode_tail does)
    constexpr uint32_t PW = (ACC_SLOTS + NW - 1) / NW;
    const uint32_t ns = acc_slots(c.quantizer);
    uint64_t x[PW];
#pragma unroll
    for (uint32_t i = 0; i < PW; ++i) {
      const uint32_t sl = wave + i * NW;
      x[i] = 0;
      if (sl < ns) x[i] = wave_sum64(acc[lane * st + sl]);       // LEAN_ROWS = 64 rows: one per lane
    }
    __syncthreads();
    if (lane == 0) {
#pragma unroll
      for (uint32_t i = 0; i < PW; ++i) if (wave + i * NW < ns) acc[wave + i * NW] = x[i];
    }
  }
  const uint32_t n_list = min(s_nlist, LISTCAP);
  const uint32_t k_rem = sg.k - above;
  uint4 me = make_uint4(0, 0, 0, 0);
  if (threadIdx.x < n_list) me = s_list[threadIdx.x];
  __syncthreads();
  bool sel = false;
  if (threadIdx.x < n_list) {
    uint32_t rank = 0;
    for (uint32_t j = 0; j < n_list; ++j) {
      const uint4 o = s_list[j];
      rank += (o.z > me.z || (o.z == me.z && o.x < me.x)) ? 1u : 0u;
    }
    sel = rank < k_rem;
    s_sel[threadIdx.x] = sel;
    if (rank == k_rem - 1) s_tau = me.z;
    if (sel) add_digits(acc, me.y, power);
  }
  __syncthreads();
  if (sel && me.z == s_tau) atomicAdd(&s_need, 1u);
  if (wave == 0) {
    const float sc = finalize_scale(acc, c.quantizer, sg.k);
    if (lane == 0) s_scale = sc;
  }
  __syncthreads();
  const UnitScale usc = unit_scale(c, s_scale, sg.k);
  uint32_t s_off = 0;
  for (uint32_t g = 0; g < wave; ++g) s_off += s_wsel[g];
  {
    uint32_t x = 0;
    for (uint32_t j = lane; j < n_list; j += WAVE) x += (s_sel[j] && s_list[j].x < d_off) ? 1u : 0u;
    s_off += wave_sum(x);
  }
  const RandKey rk1 = make_rand_key(c.seed, worker0 + w, round, 1);
  uint32_t nsent = 0;
  for (uint32_t e0 = 0; e0 < cnt_w; e0 += WAVE) {
    const uint32_t e = e0 + lane;
    const uint2 ent = ent_first;                                  // loaded one step ahead
    const uint32_t key = key_first;
    if (e + WAVE < cnt_w) { ent_first = d0[d_off + e + WAVE]; if (SPARS == QSL_RANDK) key_first = d0k[d_off + e + WAVE]; }
    uint32_t bin = 0;
    if (e < cnt_w) bin = lean_bin(SPARS == QSL_TOPK ? key_of_value(ent.y) : key, T, sh);
    bool take = e < cnt_w && bin > taubin;
    const bool maybe = e < cnt_w && bin == taubin;
    if (__ballot(maybe) != 0) {
      for (uint32_t j = 0; j < n_list; ++j) {
        const uint32_t p = s_list[j].x;
        if (maybe && p == d_off + e && s_sel[j]) take = true;
      }
    }
    const uint64_t tb = __ballot(take);
    const uint32_t pos = s_off + popc_below(tb);
    bool sent = false;
    if (take && pos < sg.k) {
      const uint64_t slot = static_cast<uint64_t>(w) * c.K + sg.koff + pos;
      sent = encode_entry(c, w, slot, ent.x, ent.y, usc, rk1, m_out, dbg_idx, dbg_level);
    }
    if (is_qsgd(c.quantizer)) {
      const uint64_t sb = __ballot(sent);
      if (sb != 0) {
        const uint32_t b_first = (sg.koff + s_off) >> 8;
        const bool in_first = ((sg.koff + pos) >> 8) == b_first;
        const uint32_t n0 = static_cast<uint32_t>(__popcll(__ballot(sent && in_first)));
        const uint32_t n1 = static_cast<uint32_t>(__popcll(sb)) - n0;
        if (lane == 0) {
          uint32_t* bc = c.blk_cnt + static_cast<uint64_t>(w) * c.QB;
          if (n0) atomicAdd(&bc[b_first], n0);
          if (n1) atomicAdd(&bc[b_first + 1], n1);
          nsent += n0 + n1;
        }
      }
    }
    s_off += static_cast<uint32_t>(__popcll(tb));
  }
  if (is_qsgd(c.quantizer) && c.L > 1 && lane == 0 && nsent) atomicAdd(&s_count, nsent);
  __syncthreads();
  if (threadIdx.x == 0) {
    usp->tau = s_tau; usp->need = s_need; usp->n_gt = sg.k - s_need; usp->scale_bits = __float_as_uint(usc.sent);
    if (is_qsgd(c.quantizer) && c.L > 1) usp->nnz = s_count;
  }
}

}  // namespace
