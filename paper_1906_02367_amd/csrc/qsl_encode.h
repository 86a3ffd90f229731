// qsl_encode.h -- From the selected coordinates to the packed message: the fp32 scale from the exact norm digits,
// encode_entry (QSGD level / sign of one selected coordinate, error update if it is transmitted) and block_encode_tail,
// which every selection path calls; k_quantize (the same for the units of the multi-pass kernels), k_surv_scan,
// k_pack (every selected coordinate is sent) and k_pack_sent (QSGD: the entries of level 0 drop out).
// Part of the single translation unit qsl.hip (included there, in this order: device, layout, select,
// encode, stream, lean, dense, decode); not a public header.
#pragma once

#include "qsl_device.h"
#include "qsl_layout.h"

namespace {

// digits -> one correctly rounded double -> the fp32 scale of the unit.  Called by all 64 lanes of a
// wave with the same arguments; lane i holds digit counter i, everything else is shuffles and ballots
// (a per-thread digit array would live in scratch memory and cost microseconds).
// The cube root by a fixed sequence of IEEE double operations (Lemma 3 with m = 3 fixes the norm, not how its root is
// rounded): 2^floor(E / 3) times 1, 2^(1/3) or 2^(2/3) for the binary exponent E of x, then eight Newton steps
// y <- (2 y + x / y^2) / 3.  x is zero or a positive normal number.
__device__ __forceinline__ double cube_root_fixed(double x) {
  if (!(x > 0.0)) return 0.0;
  const int E = static_cast<int>(static_cast<unsigned long long>(__double_as_longlong(x)) >> 52) - 1023;
  int q = E / 3, r = E % 3;
  if (r < 0) { r += 3; q -= 1; }
  double y = __longlong_as_double(static_cast<long long>(q + 1023) << 52);
  y = y * (r == 0 ? 1.0 : r == 1 ? 1.2599210498948732 : 1.5874010519681994);
  for (int it = 0; it < 8; ++it) {
    const double t = y * y;
    const double u = x / t;
    const double w = 2.0 * y;
    y = (w + u) / 3.0;
  }
  return y;
}

__device__ float finalize_scale(const uint64_t* acc, uint32_t quantizer, uint32_t k) {
  const int power = static_cast<int>(norm_power(quantizer));
  const uint32_t lane = lane_id();
  const uint64_t a = lane < acc_slots(quantizer) ? acc[lane] : 0;
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
    S = ldexp(static_cast<double>(mant), e2 - 149 * power);
  }
  if (quantizer == QSL_SIGN_L1) return static_cast<float>(S / static_cast<double>(k));           // ||v_S||_1 / k
  if (quantizer == QSL_SIGN_L2) return static_cast<float>(sqrt(S) / static_cast<double>(k));     // ||v_S||_2 / k
  if (quantizer == QSL_SIGN_L3) return static_cast<float>(cube_root_fixed(S) / static_cast<double>(k));     // ||v_S||_3 / k
  if (quantizer == QSL_SIGN_L4) return static_cast<float>(sqrt(sqrt(S)) / static_cast<double>(k));          // ||v_S||_4 / k
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
  while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (c.seg_koff[mid] <= j) lo = mid; else hi = mid; }
  return lo;
}
// segment of coordinate i: seg_dir[t] is the segment of coordinate t * 1024, so the search is over the few
// segments that touch one 1024-block instead of all L
__device__ __forceinline__ uint32_t seg_of_coord(const DevCtx& c, uint32_t i) {
  const uint32_t t = i >> 10;
  uint32_t lo = c.seg_dir[t], hi = c.seg_dir[t + 1] + 1;       // segs[lo].start <= i < segs[hi].start (or hi = L)
  while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (c.seg_start[mid] <= i) lo = mid; else hi = mid; }
  return lo;
}

__device__ __forceinline__ float qsgd_value(float N, uint32_t level, uint32_t s, bool neg) {
  const float prod = N * static_cast<float>(level);
  const float mag = prod / static_cast<float>(s);
  return neg ? -mag : mag;
}

// The scale of a unit: what the codes are computed with (the norm, or the magnitude of a sign entry) and what the
// message carries -- the same, or N / (1 + beta_{k,s}) for the scaled composition (Lemma 2).
struct UnitScale { float scale, sent; };

__device__ __forceinline__ UnitScale unit_scale(const DevCtx& c, float sc, uint32_t kl) {
  UnitScale r; r.scale = sc; r.sent = sc;
  if (c.quantizer == QSL_QSGD_SCALED) {
    const double beta = fmin(static_cast<double>(kl) / (static_cast<double>(c.s) * c.s), sqrt(static_cast<double>(kl)) / c.s);
    r.sent = sc / static_cast<float>(1.0 + beta);
  }
  return r;
}

// One selected coordinate (slot `slot` of the worker-major [R][K] arrays; coordinate idx, value bits): its code
// (QSGD: Definition 1, example 1; Sign: Definition 2), the arrays the message is packed from, the error update
// m <- v - g on a transmitted coordinate (Algorithm 1, second worker line), the optional debug outputs.
// Returns whether the coordinate is transmitted.  rk1: the random stream of the QSGD rounding.
__device__ __forceinline__ bool encode_entry(const DevCtx& c, uint32_t w, uint64_t slot, uint32_t idx, uint32_t bits,
                                             UnitScale us, const RandKey& rk1, float* m_out, uint32_t* dbg_idx,
                                             uint16_t* dbg_level) {
  const float v = __uint_as_float(bits);
  const bool neg = v < 0.0f;
  uint32_t level;
  float g;
  if (is_qsgd(c.quantizer)) {
    level = 0;
    if (us.scale > 0.0f) {
      const float a = fabsf(v) / us.scale;
      float t = a * static_cast<float>(c.s);
      if (t > static_cast<float>(c.s)) t = static_cast<float>(c.s);
      const float fl = floorf(t);
      const float frac = t - fl;
      const float r01 = static_cast<float>(rand_word(rk1, idx) >> 8) * 0x1p-24f;
      level = static_cast<uint32_t>(fl) + (r01 < frac ? 1u : 0u);
    }
    g = qsgd_value(us.sent, level, c.s, neg);
  } else if (c.quantizer == QSL_FP32) {
    level = 1;
    g = v;
  } else {
    level = 1;
    g = neg ? -us.scale : us.scale;
  }
  const bool sent = level != 0;
  if (is_qsgd(c.quantizer)) { c.sel_idx[slot] = idx; c.sel_code[slot] = level | (neg ? 0x80000000u : 0u); }   // k_pack_sent reads both
  else {                                                 // every selected coordinate is sent: nothing to compact
    c.surv_idx[slot] = idx;
    c.surv_code[slot] = c.quantizer == QSL_FP32 ? bits : (neg ? 1u : 0u);
  }
  if (sent) {
    if (idx < c.d) m_out[static_cast<uint64_t>(w) * c.d + idx] = v - g;
    else atomicOr(c.status, 2u);                       // cannot happen: a selected slot was never written
  }
  if (dbg_idx) dbg_idx[slot] = idx;
  if (dbg_level) dbg_level[slot] = static_cast<uint16_t>(level);
  return sent;
}

// What follows the ordered pass of a selection done by one block of NT threads: the block's ROWS accumulator rows
// added up, the fp32 scale, the codes and the error update of the unit's k selected coordinates (already in the
// selected arrays), the unit's state.
template <uint32_t NT, uint32_t ROWS>
__device__ void block_encode_tail(const DevCtx& c, const SegInfo& sg, uint32_t w, uint64_t u, uint32_t tau, uint32_t need,
                                  uint32_t worker0, uint64_t round, float* m_out, uint32_t* dbg_idx, uint16_t* dbg_level,
                                  uint64_t* acc, float* s_scale, uint32_t* s_count) {
  constexpr uint32_t NW = NT / 64, PW = (ACC_SLOTS + NW - 1) / NW;      // digit counters per wave
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t* oi = c.sel_idx + static_cast<uint64_t>(w) * c.K + sg.koff;
  const uint32_t* ov = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff;
  __syncthreads();                                   // the selected arrays and the accumulator rows are complete
  uint64_t x[PW];
#pragma unroll
  for (uint32_t i = 0; i < PW; ++i) {
    const uint32_t s = wave + i * NW;                // wave-uniform
    x[i] = 0;
    if (s < acc_slots(c.quantizer)) x[i] = wave_sum64(lane < ROWS ? acc[lane * acc_stride(c.quantizer) + s] : 0);
  }
  __syncthreads();
  if (lane == 0) {
#pragma unroll
    for (uint32_t i = 0; i < PW; ++i) if (wave + i * NW < acc_slots(c.quantizer)) acc[wave + i * NW] = x[i];
  }
  if (threadIdx.x == 0) *s_count = 0;
  __syncthreads();
  if (wave == 0) {
    const float sc = finalize_scale(acc, c.quantizer, sg.k);
    if (lane == 0) *s_scale = sc;
  }
  __syncthreads();
  const UnitScale usc = unit_scale(c, *s_scale, sg.k);
  const RandKey rk1 = make_rand_key(c.seed, worker0 + w, round, 1);
  uint32_t nsent = 0;
  for (uint32_t j = threadIdx.x; j < sg.k; j += NT) {
    const uint64_t slot = static_cast<uint64_t>(w) * c.K + sg.koff + j;
    const bool sent = encode_entry(c, w, slot, oi[j], ov[j], usc, rk1, m_out, dbg_idx, dbg_level);
    if (sent && is_qsgd(c.quantizer)) { atomicAdd(&c.blk_cnt[static_cast<uint64_t>(w) * c.QB + ((sg.koff + j) >> 8)], 1u); ++nsent; }
  }
  if (is_qsgd(c.quantizer) && c.L > 1) {              // the unit's entry count for the message header
    nsent = wave_sum(nsent);
    if (lane == 0 && nsent) atomicAdd(s_count, nsent);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    UnitState* usp = &c.units[u];
    usp->tau = tau; usp->need = need; usp->n_gt = sg.k - need; usp->scale_bits = __float_as_uint(usc.sent);
    if (is_qsgd(c.quantizer) && c.L > 1) usp->nnz = *s_count;
  }
}

// The units that k_lean_emit has already encoded are skipped here: a guessing unit, unless its guess failed and
// the multi-pass kernels of this call took it over (`safe`).
__global__ __launch_bounds__(BLOCK) void k_quantize(DevCtx c, float* m_out, uint32_t worker0, uint64_t round,
                                                    uint32_t* dbg_idx, uint16_t* dbg_level, int safe) {
  __shared__ uint32_t s_w[BLOCK / 64];
  __shared__ float s_scale[BLOCK];
  __shared__ uint32_t s_mine[BLOCK];
  const uint32_t w = blockIdx.y;
  const uint32_t j = blockIdx.x * BLOCK + threadIdx.x;
  // the scales of the units this block's slots belong to (at most one unit per slot)
  const uint32_t j_first = blockIdx.x * BLOCK, j_last = min(j_first + BLOCK, c.K) - 1;
  const uint32_t seg_first = c.L == 1 ? 0u : seg_of_slot(c, j_first);
  const uint32_t seg_last = c.L == 1 ? 0u : seg_of_slot(c, j_last);
  for (uint32_t i = threadIdx.x >> 6; i <= seg_last - seg_first; i += BLOCK / 64) {     // a wave per unit
    const uint32_t seg = seg_first + i;
    const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
    const UnitState us = c.units[u];
    const bool mine = us.path != PATH_SMALL && !(us.path == PATH_FAST && !(safe && us.fell_back));
    float sc = 0.0f;
    if (mine) sc = finalize_scale(c.norm_acc + u * ACC_SLOTS, c.quantizer, c.segs[seg].k);
    if (lane_id() == 0) {
      s_scale[i] = sc;
      s_mine[i] = mine;
      // the block holding the unit's first slot records what the message carries
      if (mine && c.segs[seg].koff >= j_first) c.units[u].scale_bits = __float_as_uint(unit_scale(c, sc, c.segs[seg].k).sent);
    }
  }
  __syncthreads();
  bool sent = false;
  if (j < c.K) {
    const uint32_t seg = c.L == 1 ? 0u : seg_of_slot(c, j);
    if (s_mine[seg - seg_first]) {
      const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
      const uint64_t slot = static_cast<uint64_t>(w) * c.K + j;
      const RandKey rk1 = make_rand_key(c.seed, worker0 + w, round, 1);
      sent = encode_entry(c, w, slot, c.sel_idx[slot], c.sel_val[slot], unit_scale(c, s_scale[seg - seg_first], c.segs[seg].k),
                          rk1, m_out, dbg_idx, dbg_level);
      if (sent && is_qsgd(c.quantizer) && c.L > 1) atomicAdd(&c.units[u].nnz, 1u);
    }
  }
  if (!is_qsgd(c.quantizer)) return;                       // survivors are counted only where some may drop out
  const uint32_t wc = __popcll(__ballot(sent));
  if (lane_id() == 0) s_w[threadIdx.x >> 6] = wc;
  __syncthreads();
  uint32_t* cnt = c.blk_cnt + static_cast<uint64_t>(w) * c.QB;
  // a block of 256 slots may also hold entries that another kernel encodes: the counts are added (they start at zero)
  if (threadIdx.x == 0) {
    const uint32_t n = s_w[0] + s_w[1] + s_w[2] + s_w[3];
    if (n) atomicAdd(&cnt[blockIdx.x], n);
  }
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

// The last kernel of a call also returns the shared scratch of its worker to all-zero; the blocks of worker w share the work.
__device__ __forceinline__ void end_of_call(const DevCtx& c, uint32_t w, uint32_t nzero) {
  {
    const uint64_t tid = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x, nth = static_cast<uint64_t>(gridDim.x) * BLOCK;
    // histograms: only the first `nzero` of the segments that have any (the units of the multi-pass kernels; the
    // guessing units too when those kernels stood by for them in this call), and of the third digit only its 256 bins
    constexpr uint32_t ZW = 2 * HBINS + 256;
    uint32_t* h = c.hist + static_cast<uint64_t>(w) * c.L * 3 * HBINS;
    for (uint64_t i = tid; i < static_cast<uint64_t>(nzero) * ZW; i += nth)
      h[static_cast<uint64_t>(c.big_segs[i / ZW]) * 3 * HBINS + i % ZW] = 0;
    uint32_t* ct = c.ctr + static_cast<uint64_t>(w) * c.L * CTR_LINES * PAD;                 // counters: the guessing segments only
    for (uint64_t i = tid; i < static_cast<uint64_t>(c.nfast) * CTR_LINES; i += nth)
      ct[(static_cast<uint64_t>(c.fast_segs[i / CTR_LINES]) * CTR_LINES + i % CTR_LINES) * PAD] = 0;
    uint64_t* na = c.norm_acc + static_cast<uint64_t>(w) * c.L * ACC_SLOTS;
    const uint32_t ns = acc_slots(c.quantizer);
    for (uint64_t i = tid; i < static_cast<uint64_t>(c.L) * ns; i += nth) na[(i / ns) * ACC_SLOTS + i % ns] = 0;
    // the next call's counters of transmitted entries (the other of the two arrays; nobody uses it during this call)
    {
      const uint64_t gtid = (static_cast<uint64_t>(w) * gridDim.x + blockIdx.x) * BLOCK + threadIdx.x;
      const uint64_t gnth = static_cast<uint64_t>(gridDim.y) * gridDim.x * BLOCK;
      for (uint64_t i = gtid; i < static_cast<uint64_t>(c.Rmax) * c.QB; i += gnth) c.blk_cnt_next[i] = 0;
    }
    // ... and the guess that this call's candidates suggest becomes the next call's
    if (c.sparsifier == QSL_TOPK)
      for (uint64_t i = tid; i < c.nfast; i += nth) {
        UnitState* us = &c.units[static_cast<uint64_t>(w) * c.L + c.fast_segs[i]];
        us->T_used = us->T; us->T = us->T_next; us->sh = us->sh_next;
      }
  }
}

__global__ __launch_bounds__(BLOCK) void k_pack(DevCtx c, uint8_t* msg, uint64_t* msg_bits, uint32_t nzero) {
  const uint32_t w = blockIdx.y;
  end_of_call(c, w, nzero);
  const uint64_t nnz = c.K;                          // a quantiser that sends every selected coordinate (QSGD: k_pack_sent)
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L);
  const uint64_t idx_words = (nnz * c.w_idx + 31) / 32, code_words = (nnz * c.w_val + 31) / 32;
  // one word per thread, or several a grid's width apart (the host sizes the grid)
  for (uint64_t q = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x; q < c.cap_words; q += static_cast<uint64_t>(gridDim.x) * BLOCK) {
    uint32_t word = 0;
    if (q == 0) word = static_cast<uint32_t>(nnz);
    else if (q < 1 + static_cast<uint64_t>(c.L)) word = c.units[static_cast<uint64_t>(w) * c.L + (q - 1)].scale_bits;
    else if (q < hdr + idx_words) word = gather_word(c.surv_idx + static_cast<uint64_t>(w) * c.K, nnz, c.w_idx, q - hdr);
    else if (q < hdr + idx_words + code_words)
      word = gather_word(c.surv_code + static_cast<uint64_t>(w) * c.K, nnz, c.w_val, q - hdr - idx_words);
    reinterpret_cast<uint32_t*>(msg + static_cast<uint64_t>(w) * c.cap_words * 4)[q] = word;
    if (q == 0 && msg_bits) msg_bits[w] = hdr * 32 + nnz * (c.w_idx + c.w_val);
  }
}

// QSGD drops the entries it rounds to level 0.  k_pack_sent puts the message together from the selected arrays as they
// are, with no compacted copy in between: block b takes the 256 slots b * 256 .. b * 256 + 255, lines up its transmitted
// entries in LDS, and writes their index and code fields where they belong -- behind those of the blocks before it (it
// adds up their counts itself).  The words that lie wholly inside the block's share of a section are stored; the two at
// its ends, which it may share with its neighbours, are added with atomicOr to words that k_stream has cleared
// (as it has the padding behind the last field).
__device__ __forceinline__ void put_fields(uint32_t* words, uint64_t bit0, const uint32_t* s_val, uint32_t n, uint32_t width) {
  if (n == 0 || width == 0) return;
  const uint64_t bit_end = bit0 + static_cast<uint64_t>(n) * width;              // the block's fields: bits [bit0, bit_end)
  const uint64_t q_lo = bit0 >> 5, q_hi = (bit_end - 1) >> 5;
  for (uint64_t q = q_lo + threadIdx.x; q <= q_hi; q += BLOCK) {
    const uint64_t b_lo = max(q * 32, bit0), b_hi = min(q * 32 + 32, bit_end);   // the part of word q that is the block's
    uint32_t out = 0;
    for (uint64_t e = (b_lo - bit0) / width; e * width + bit0 < b_hi; ++e) {     // fields that overlap the word
      const int64_t sh = static_cast<int64_t>(bit0 + e * width) - static_cast<int64_t>(q * 32);
      const uint32_t f = s_val[e];
      out |= sh >= 0 ? (f << sh) : (f >> (-sh));
    }
    if (b_lo == q * 32 && b_hi == q * 32 + 32) words[q] = out;
    else if (out) atomicOr(&words[q], out);
  }
}

__global__ __launch_bounds__(BLOCK) void k_pack_sent(DevCtx c, uint8_t* msg, uint64_t* msg_bits, uint32_t nzero) {
  __shared__ uint32_t s_idx[BLOCK], s_code[BLOCK], s_w[BLOCK / 64], s_part[4];
  const uint32_t w = blockIdx.y, b = blockIdx.x, lane = lane_id(), wave = threadIdx.x >> 6;
  end_of_call(c, w, nzero);
  // transmitted entries before this block, and in all
  uint32_t before, nnz;
  if (c.QB > MAX_QB_INLINE) {
    before = c.blk_pre[static_cast<uint64_t>(w) * (c.QB + 1) + b]; nnz = c.blk_pre[static_cast<uint64_t>(w) * (c.QB + 1) + c.QB];
  } else {
    const uint32_t* cnt = c.blk_cnt + static_cast<uint64_t>(w) * c.QB;
    uint32_t x = 0, y = 0;
    for (uint32_t i = threadIdx.x; i < c.QB; i += BLOCK) { const uint32_t v = cnt[i]; y += v; if (i < b) x += v; }
    x = wave_sum(x); y = wave_sum(y);
    if (lane == 0) { s_w[wave] = x; s_part[wave] = y; }
    __syncthreads();
    before = s_w[0] + s_w[1] + s_w[2] + s_w[3]; nnz = s_part[0] + s_part[1] + s_part[2] + s_part[3];
    __syncthreads();
  }
  // the block's transmitted entries, in slot order, side by side in LDS
  const uint32_t j = b * BLOCK + threadIdx.x;
  const uint64_t slot = static_cast<uint64_t>(w) * c.K + j;
  const uint32_t code = j < c.K ? c.sel_code[slot] : 0u;
  const bool sent = (code & 0x7FFFFFFFu) != 0;
  const uint64_t bal = __ballot(sent);
  if (lane == 0) s_w[wave] = static_cast<uint32_t>(__popcll(bal));
  __syncthreads();
  uint32_t pos = popc_below(bal);
  for (uint32_t i = 0; i < wave; ++i) pos += s_w[i];
  const uint32_t n = s_w[0] + s_w[1] + s_w[2] + s_w[3];
  if (sent) {
    s_idx[pos] = c.sel_idx[slot];
    s_code[pos] = ((code & 0x7FFFFFFFu) - 1u) | ((code >> 31) << c.w_lev);      // a level 1..s is written as level - 1
  }
  __syncthreads();
  uint32_t* words = reinterpret_cast<uint32_t*>(msg + static_cast<uint64_t>(w) * c.cap_words * 4);
  const bool counts = c.L > 1;
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L) + (counts ? c.L : 0);
  const uint64_t idx_words = (static_cast<uint64_t>(nnz) * c.w_idx + 31) / 32;
  put_fields(words, hdr * 32 + static_cast<uint64_t>(before) * c.w_idx, s_idx, n, c.w_idx);
  put_fields(words, (hdr + idx_words) * 32 + static_cast<uint64_t>(before) * c.w_val, s_code, n, c.w_val);
  if (b == 0) {                                        // the header: entry count, scales, entry counts of the segments
    for (uint64_t q = threadIdx.x; q < hdr; q += BLOCK)
      words[q] = q == 0 ? nnz : q < 1 + static_cast<uint64_t>(c.L) ? c.units[static_cast<uint64_t>(w) * c.L + (q - 1)].scale_bits
                                                                   : c.units[static_cast<uint64_t>(w) * c.L + (q - 1 - c.L)].nnz;
    if (threadIdx.x == 0 && msg_bits) msg_bits[w] = hdr * 32 + static_cast<uint64_t>(nnz) * (c.w_idx + c.w_val);
  }
}

}  // namespace
