// qsl_dense.h -- An operator that keeps every coordinate (k = size in every segment: the error-feedback schemes
// without sparsification that Section 5 compares with, as this operator) with the index-free message format: two
// streaming passes and nothing per entry in between.
//   k_dense_norm    v = m + Delta (Algorithm 1, first worker line) written over the error memory, 12 bytes per
//                   coordinate, with the exact digits of every segment's norm added up on the way
//   k_dense_sum     the digit sums that the blocks of k_dense_norm stored, into their units' counters
//   k_dense_scales  one wave per unit: digits -> fp32 scale (||v||_2 for QSGD, ||v||_1 / k or ||v||_2 / k for Sign)
//   k_dense_encode  reads v, writes m' = v - g (second worker line) and the packed codes, 8 bytes per coordinate:
//                   a block owns 4096 consecutive coordinates and with them whole 32-bit words of the code stream
// Part of the single translation unit qsl.hip (included after qsl_encode.h); not a public header.
#pragma once

#include "qsl_device.h"
#include "qsl_layout.h"
#include "qsl_select.h"
#include "qsl_encode.h"

namespace {

constexpr uint32_t DTILE = 4096;             // coordinates per tile: 256 threads x 4 x dwordx4
// Blocks per worker of the first pass, each a contiguous range of tiles.  The pass wants many: without the digits
// (fp32 values, 2 x 25.6 M coordinates) 1024 blocks per worker take 127 us, 2048 121 us, 4096 112 us, 16384 100 us.  With
// that many, adding every block's digits to its unit's counters by atomics costs more than it saves (292 us: additions
// to one address queue up), so a block stores the sums of its first unit as a row of its own and k_dense_sum adds the
// rows up; only what a block meets beyond its first unit (few blocks, if any) goes to the counters directly.
constexpr uint32_t MAX_DENSE_BLOCKS = 16384;
constexpr uint32_t NO_UNIT = 0xFFFFFFFFu;
constexpr uint32_t MAX_ENCODE_BLOCKS = 8192; // ... and of the second, which has no such ending

// digits of |v| (or v^2) straight into a unit's counters in memory (for the few tiles that span several segments)
__device__ __forceinline__ void add_digits_global(uint64_t* acc, uint32_t bits, uint32_t power) {
  const uint32_t ab = bits & 0x7FFFFFFFu;
  const uint32_t ex = ab >> 23, frac = ab & 0x7FFFFFu;
  const uint32_t M = ex ? (frac | 0x800000u) : frac;
  const uint32_t e1 = ex ? ex : 1u;
  if (M == 0) return;
  auto add = [&](uint32_t q, uint64_t x) { if (x) atomicAdd(reinterpret_cast<unsigned long long*>(acc + q), static_cast<unsigned long long>(x)); };
  uint64_t lo, hi;                                         // M^power < 2^96
  power_of_mantissa(M, power, &lo, &hi);
  const uint32_t p = power * (e1 - 1u), q = p >> 5, r = p & 31u;
  const uint64_t a0 = lo << r;
  const uint64_t a1 = (hi << r) | (r ? lo >> (64 - r) : 0);
  add(q, a0 & 0xFFFFFFFFu); add(q + 1, a0 >> 32); add(q + 2, a1 & 0xFFFFFFFFu); add(q + 3, a1 >> 32);
}

// the tiles [t_lo, t_hi) of block b out of nb
__device__ __forceinline__ void dense_range(uint64_t d, uint32_t b, uint32_t nb, uint64_t* t_lo, uint64_t* t_hi) {
  const uint64_t ntiles = (d + DTILE - 1) / DTILE;
  *t_lo = ntiles * b / nb; *t_hi = ntiles * (b + 1) / nb;
}

// With `xm` given, `delta` holds the local models and Delta = xm - delta is formed on the fly (as in k_stream).
template <bool DIFF>
__global__ __launch_bounds__(BLOCK) void k_dense_norm(DevCtx c, const float* m, const float* delta, const float* xm,
                                                      float* m_out) {
  __shared__ uint64_t acc[ACC_ROWS * (ACC_SLOTS + 1)];
  const uint32_t w = blockIdx.y, wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t power = norm_power(c.quantizer);
  const bool need_norm = c.quantizer != QSL_FP32;
  uint64_t* mine = acc + (wave * 8 + (lane & 7u)) * acc_stride(c.quantizer);
  for (uint32_t i = threadIdx.x; i < ACC_ROWS * acc_stride(c.quantizer); i += BLOCK) acc[i] = 0;
  __syncthreads();
  const uint64_t row = static_cast<uint64_t>(w) * c.d;
  uint64_t t_lo, t_hi;
  dense_range(c.d, blockIdx.x, gridDim.x, &t_lo, &t_hi);
  uint32_t cur = NO_UNIT;                           // the segment whose digits the block's rows hold
  bool nonfinite = false;
  bool own_row = true;                              // nothing stored yet: the next sums go to the block's own row
  const uint64_t nb = gridDim.x;
  // the rows added up: into the block's own row the first time, into the segment's counters after that; then zero again
  // (uniform over the block)
  auto flush = [&]() {
    __syncthreads();
    if (cur != NO_UNIT) {
      uint64_t* ga = c.norm_acc + (static_cast<uint64_t>(w) * c.L + cur) * ACC_SLOTS;
      for (uint32_t s = wave; s < acc_slots(c.quantizer); s += BLOCK / 64) {
        uint64_t x = lane < ACC_ROWS ? acc[lane * acc_stride(c.quantizer) + s] : 0;
        x = wave_sum64(x);
        if (lane == 0) {
          if (own_row) c.dense_part[(static_cast<uint64_t>(w) * ACC_SLOTS + s) * nb + blockIdx.x] = x;
          else if (x) atomicAdd(reinterpret_cast<unsigned long long*>(ga + s), static_cast<unsigned long long>(x));
        }
      }
      if (own_row && threadIdx.x == 0) c.dense_tag[static_cast<uint64_t>(w) * nb + blockIdx.x] = cur;
      own_row = false;
      __syncthreads();
      for (uint32_t i = threadIdx.x; i < ACC_ROWS * acc_stride(c.quantizer); i += BLOCK) acc[i] = 0;
      __syncthreads();
    }
  };
  for (uint64_t tile = t_lo; tile < t_hi; ++tile) {
    const uint64_t base = tile * DTILE;
    f4u v[4];
    // the tile's loads first, then its stores (146 us against 159 us one group of four at a time, 2 x 25.6 M coordinates in
    // 1024 blocks per worker; the next tile's loads issued before this tile's digits are added: no change)
    if (base + DTILE <= c.d) {
      f4u a[4], b[4], x[4];
#pragma unroll
      for (uint32_t q = 0; q < 4; ++q) {
        const uint64_t e = base + q * 1024 + threadIdx.x * 4;
        a[q] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(m + row + e));
        b[q] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(delta + row + e));
        if (DIFF) x[q] = *reinterpret_cast<const f4u*>(xm + e);
      }
#pragma unroll
      for (uint32_t q = 0; q < 4; ++q) {
        const uint64_t e = base + q * 1024 + threadIdx.x * 4;
        if (DIFF) b[q] = x[q] - b[q];
        v[q] = a[q] + b[q];
        __builtin_nontemporal_store(v[q], reinterpret_cast<f4u*>(m_out + row + e));
      }
    } else {                                        // the row's last, ragged tile
#pragma unroll
      for (uint32_t q = 0; q < 4; ++q) {
        const uint64_t e = base + q * 1024 + threadIdx.x * 4;
        v[q] = f4u{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j)
          if (e + j < c.d) {
            const float dl = DIFF ? xm[e + j] - delta[row + e + j] : delta[row + e + j];
            v[q][j] = m[row + e + j] + dl;
            m_out[row + e + j] = v[q][j];
          }
      }
    }
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) nonfinite |= (__float_as_uint(v[q][j]) & 0x7FFFFFFFu) >= 0x7F800000u;
    }
    if (!need_norm) continue;
    const uint64_t last = min(base + DTILE, c.d) - 1;
    const uint32_t seg_first = c.L == 1 ? 0u : seg_of_coord(c, static_cast<uint32_t>(base));
    const uint32_t seg_last = c.L == 1 ? 0u : seg_of_coord(c, static_cast<uint32_t>(last));
    if (seg_first == seg_last) {
      if (seg_first != cur) { flush(); cur = seg_first; }
#pragma unroll
      for (uint32_t q = 0; q < 4; ++q) {
        const uint64_t e = base + q * 1024 + threadIdx.x * 4;
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) if (e + j < c.d) add_digits(mine, __float_as_uint(v[q][j]), power);
      }
    } else {                                          // several segments in one tile: each coordinate to its own unit's counters
      flush(); cur = NO_UNIT;
#pragma unroll
      for (uint32_t q = 0; q < 4; ++q) {
        const uint64_t e = base + q * 1024 + threadIdx.x * 4;
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j)
          if (e + j < c.d) {
            const uint32_t seg = seg_of_coord(c, static_cast<uint32_t>(e + j));
            add_digits_global(c.norm_acc + (static_cast<uint64_t>(w) * c.L + seg) * ACC_SLOTS, __float_as_uint(v[q][j]), power);
          }
      }
    }
  }
  flush();
  if (own_row && threadIdx.x == 0) c.dense_tag[static_cast<uint64_t>(w) * nb + blockIdx.x] = NO_UNIT;   // no row from this block
  if (__ballot(nonfinite) != 0 && lane == 0) atomicOr(c.status, 1u);
}

// The rows of k_dense_norm's blocks into the counters of their units.  A block takes 512 rows, each of its waves one digit
// (or two, or three): a lane adds up its eight rows' sums of that digit, the wave its lanes', and one lane adds the result
// to the unit's counter -- if the 512 rows belong to one unit, as they nearly always do; else every row goes to its own
// unit's counters.  (A thread per row and a wave-wide sum per digit: 14 us for 2 x 6240 rows; this way 4.5 us.)
constexpr uint32_t SUM_BLOCK = 1024, SUM_ROWS = 512;
__global__ __launch_bounds__(SUM_BLOCK) void k_dense_sum(DevCtx c, uint32_t nb) {
  constexpr uint32_t G = SUM_ROWS / 64;
  const uint32_t w = blockIdx.y, lane = lane_id(), wave = threadIdx.x >> 6;
  const uint32_t r0 = blockIdx.x * SUM_ROWS;
  uint32_t tags[G];
#pragma unroll
  for (uint32_t g = 0; g < G; ++g) {
    const uint32_t b = r0 + g * 64 + lane;
    tags[g] = b < nb ? c.dense_tag[static_cast<uint64_t>(w) * nb + b] : NO_UNIT;
  }
  uint32_t tag0 = NO_UNIT;                           // the unit of the first row that has one (every wave finds the same)
#pragma unroll
  for (uint32_t g = 0; g < G; ++g) {
    const uint64_t bal = __ballot(tags[g] != NO_UNIT);
    if (tag0 == NO_UNIT && bal != 0) tag0 = __shfl(tags[g], __ffsll(static_cast<long long>(bal)) - 1, WAVE);
  }
  if (tag0 == NO_UNIT) return;
  bool mixed = false;
#pragma unroll
  for (uint32_t g = 0; g < G; ++g) mixed = mixed || __ballot(tags[g] != NO_UNIT && tags[g] != tag0) != 0;
  for (uint32_t s = wave; s < acc_slots(c.quantizer); s += SUM_BLOCK / 64) {
    uint64_t x[G];
#pragma unroll
    for (uint32_t g = 0; g < G; ++g)
      x[g] = tags[g] != NO_UNIT ? c.dense_part[(static_cast<uint64_t>(w) * ACC_SLOTS + s) * nb + r0 + g * 64 + lane] : 0;
    if (!mixed) {
      uint64_t sum = 0;
#pragma unroll
      for (uint32_t g = 0; g < G; ++g) sum += x[g];
      sum = wave_sum64(sum);
      if (lane == 0 && sum)
        atomicAdd(reinterpret_cast<unsigned long long*>(c.norm_acc + (static_cast<uint64_t>(w) * c.L + tag0) * ACC_SLOTS + s),
                  static_cast<unsigned long long>(sum));
    } else {
#pragma unroll
      for (uint32_t g = 0; g < G; ++g)
        if (x[g]) atomicAdd(reinterpret_cast<unsigned long long*>(c.norm_acc + (static_cast<uint64_t>(w) * c.L + tags[g]) * ACC_SLOTS + s),
                            static_cast<unsigned long long>(x[g]));
    }
  }
}

// one wave per unit: the scale the codes are computed with and the scale the message carries; the digit counters
// are returned to zero for the next call
__global__ __launch_bounds__(BLOCK) void k_dense_scales(DevCtx c, uint32_t U) {
  const uint32_t u = blockIdx.x * (BLOCK / 64) + (threadIdx.x >> 6);
  if (u >= U) return;
  const uint32_t seg = u % c.L, lane = lane_id();
  const uint32_t kl = c.segs[seg].k;
  const float sc = finalize_scale(c.norm_acc + static_cast<uint64_t>(u) * ACC_SLOTS, c.quantizer, kl);
  if (lane < ACC_SLOTS) c.norm_acc[static_cast<uint64_t>(u) * ACC_SLOTS + lane] = 0;
  if (lane == 0) {
    const UnitScale us = unit_scale(c, sc, kl);
    c.units[u].scale_code = __float_as_uint(us.scale);
    c.units[u].scale_bits = __float_as_uint(us.sent);
    c.units[u].cand = 0; c.units[u].fell_back = 0; c.units[u].tau = 0; c.units[u].need = 0; c.units[u].n_gt = kl; c.units[u].nnz = kl;
  }
}

__global__ __launch_bounds__(BLOCK) void k_dense_encode(DevCtx c, float* m_out, uint32_t worker0, uint64_t round, uint8_t* msg,
                                                        uint64_t* msg_bits, uint32_t* dbg_idx, uint16_t* dbg_level) {
  __shared__ uint32_t s_bits[(DTILE / 32) * 32];        // the tile's part of the code stream: 128 words per bit of code width
  const uint32_t w = blockIdx.y;
  const uint32_t wv = c.w_val;
  uint32_t* words = reinterpret_cast<uint32_t*>(msg + static_cast<uint64_t>(w) * c.cap_words * 4);
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L);
  const uint64_t code_words = (c.d * wv + 31) / 32;
  if (blockIdx.x == 0) {                               // header: the length word, the scales; the payload bit count
    for (uint64_t i = threadIdx.x; i < hdr; i += BLOCK)
      words[i] = i == 0 ? static_cast<uint32_t>(c.d) : c.units[static_cast<uint64_t>(w) * c.L + (i - 1)].scale_bits;
    if (threadIdx.x == 0 && msg_bits) msg_bits[w] = hdr * 32 + c.d * wv;
  }
  if (blockIdx.x == gridDim.x - 1)                     // zero padding up to the capacity
    for (uint64_t i = hdr + code_words + threadIdx.x; i < c.cap_words; i += BLOCK) words[i] = 0;
  const uint64_t row = static_cast<uint64_t>(w) * c.d;
  const RandKey rk1 = make_rand_key(c.seed, worker0 + w, round, 1);
  uint64_t t_lo, t_hi;
  dense_range(c.d, blockIdx.x, gridDim.x, &t_lo, &t_hi);
  uint32_t cur = 0xFFFFFFFFu;
  float cur_scale = 0.f, cur_sent = 0.f;
  for (uint64_t tile = t_lo; tile < t_hi; ++tile) {
    const uint64_t base = tile * DTILE;
    const uint64_t last = min(base + DTILE, c.d) - 1;
    const uint32_t seg_first = c.L == 1 ? 0u : seg_of_coord(c, static_cast<uint32_t>(base));
    const uint32_t seg_last = c.L == 1 ? 0u : seg_of_coord(c, static_cast<uint32_t>(last));
    const bool one_seg = seg_first == seg_last;
    if (one_seg && seg_first != cur) {
      cur = seg_first;
      const UnitState& us = c.units[static_cast<uint64_t>(w) * c.L + cur];
      cur_scale = __uint_as_float(us.scale_code); cur_sent = __uint_as_float(us.scale_bits);
    }
    for (uint32_t i = threadIdx.x; i < (DTILE / 32) * wv; i += BLOCK) s_bits[i] = 0;
    __syncthreads();
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      const uint32_t le = q * 1024 + threadIdx.x * 4;           // inside the tile
      const uint64_t e = base + le;
      if (e >= c.d) continue;
      f4u x = {0.f, 0.f, 0.f, 0.f};
      const bool whole = e + 4 <= c.d;
      if (whole) x = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(m_out + row + e));
      else {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) if (e + j < c.d) x[j] = m_out[row + e + j];
      }
      Words4 rw = {{0u, 0u, 0u, 0u}};
      if (is_qsgd(c.quantizer)) rw = rand_words4(rk1, static_cast<uint32_t>(e));     // e is a multiple of 4: one block
      f4u res = x;
      uint32_t code[4];
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) {
        float scale = cur_scale, sent_scale = cur_sent;
        if (!one_seg && e + j < c.d) {
          const UnitState& us = c.units[static_cast<uint64_t>(w) * c.L + seg_of_coord(c, static_cast<uint32_t>(e + j))];
          scale = __uint_as_float(us.scale_code); sent_scale = __uint_as_float(us.scale_bits);
        }
        const float v = x[j];
        const bool neg = v < 0.0f;
        uint32_t level = 1;
        float g;
        if (is_qsgd(c.quantizer)) {                      // Definition 1, example 1: the same single IEEE operations as encode_entry
          level = 0;
          if (scale > 0.0f) {
            const float a = fabsf(v) / scale;
            float t = a * static_cast<float>(c.s);
            if (t > static_cast<float>(c.s)) t = static_cast<float>(c.s);
            const float fl = floorf(t);
            const float frac = t - fl;
            const float r01 = static_cast<float>(rw.w[j] >> 8) * 0x1p-24f;
            level = static_cast<uint32_t>(fl) + (r01 < frac ? 1u : 0u);
          }
          g = qsgd_value(sent_scale, level, c.s, neg);
          code[j] = level | (static_cast<uint32_t>(neg) << c.w_lev);
        } else if (c.quantizer == QSL_FP32) {
          g = v; code[j] = __float_as_uint(v);
        } else {                                         // Definition 2
          g = neg ? -scale : scale; code[j] = neg;
        }
        if (level != 0) res[j] = v - g;                  // Algorithm 1, second worker line
        if (e + j < c.d) {
          if (dbg_idx) dbg_idx[static_cast<uint64_t>(w) * c.K + e + j] = static_cast<uint32_t>(e + j);
          if (dbg_level) dbg_level[static_cast<uint64_t>(w) * c.K + e + j] = static_cast<uint16_t>(level);
        } else code[j] = 0;
      }
      if (whole) __builtin_nontemporal_store(res, reinterpret_cast<f4u*>(m_out + row + e));
      else {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) if (e + j < c.d) m_out[row + e + j] = res[j];
      }
      // the four codes into the tile's bit buffer
      if (wv == 32) {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) s_bits[le + j] = code[j];
      } else if (wv <= 16) {
        const uint64_t val = static_cast<uint64_t>(code[0]) | (static_cast<uint64_t>(code[1]) << wv) |
                             (static_cast<uint64_t>(code[2]) << (2 * wv)) | (static_cast<uint64_t>(code[3]) << (3 * wv));
        const uint32_t o = le * wv, word = o >> 5, sh = o & 31u;
        const uint64_t lo = val << sh;
        if (static_cast<uint32_t>(lo)) atomicOr(&s_bits[word], static_cast<uint32_t>(lo));
        if (lo >> 32) atomicOr(&s_bits[word + 1], static_cast<uint32_t>(lo >> 32));
        if (sh && (val >> (64 - sh))) atomicOr(&s_bits[word + 2], static_cast<uint32_t>(val >> (64 - sh)));
      } else {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
          const uint32_t o = (le + j) * wv, word = o >> 5, sh = o & 31u;
          const uint64_t lo = static_cast<uint64_t>(code[j]) << sh;
          if (static_cast<uint32_t>(lo)) atomicOr(&s_bits[word], static_cast<uint32_t>(lo));
          if (lo >> 32) atomicOr(&s_bits[word + 1], static_cast<uint32_t>(lo >> 32));
        }
      }
    }
    __syncthreads();
    const uint64_t w0 = tile * (DTILE / 32) * wv;        // the tile's first word of the code stream
    for (uint32_t i = threadIdx.x; i < (DTILE / 32) * wv; i += BLOCK)
      if (w0 + i < code_words) words[hdr + w0 + i] = s_bits[i];
    __syncthreads();
  }
}

}  // namespace
