// Device-side helpers shared by the kernels of the compression library: wavefront (64-lane)
// reductions and scans, the Philox4x32-10 counter-based generator, message bit-field access.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qsl {

constexpr uint32_t WAVE = 64;

// four floats / two 32-bit words that need only 4-byte alignment: rows of an [R, d] array and
// the segments inside a row start at arbitrary coordinates; gfx950 serves unaligned dwordx4 accesses
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u2a __attribute__((ext_vector_type(2), aligned(8)));

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (WAVE - 1); }

// number of set bits of `mask` in lanes below the caller's
__device__ __forceinline__ uint32_t popc_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, WAVE);
  return x;
}

__device__ __forceinline__ uint64_t wave_sum64(uint64_t x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t lo = __shfl_xor(static_cast<uint32_t>(x), o, WAVE);
    const uint32_t hi = __shfl_xor(static_cast<uint32_t>(x >> 32), o, WAVE);
    x += (static_cast<uint64_t>(hi) << 32) | lo;
  }
  return x;
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint64_t wave_inclusive_scan64(uint64_t x) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t lo = __shfl_up(static_cast<uint32_t>(x), o, WAVE);
    const uint32_t hi = __shfl_up(static_cast<uint32_t>(x >> 32), o, WAVE);
    if (lane_id() >= static_cast<uint32_t>(o)) x += (static_cast<uint64_t>(hi) << 32) | lo;
  }
  return x;
}

// Exclusive prefix sum over a block of up to 1024 threads (blockDim.x a multiple of 64).
// `scratch` holds at least 17 uint64.  Returns the exclusive prefix of x; *total = block sum.
__device__ __forceinline__ uint64_t block_exclusive_scan64(uint64_t x, uint64_t* scratch, uint64_t* total) {
  const uint32_t wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const uint64_t inc = wave_inclusive_scan64(x);
  __syncthreads();                       // scratch may still be read from a previous call
  if (lane_id() == 63) scratch[wave] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint64_t run = 0;
    for (uint32_t i = 0; i < nw; ++i) { const uint64_t t = scratch[i]; scratch[i] = run; run += t; }
    scratch[16] = run;
  }
  __syncthreads();
  *total = scratch[16];
  return scratch[wave] + inc - x;
}

// Philox4x32 with ten rounds (Salmon, Moraes, Dror, Shaw, SC'11).
struct Words4 { uint32_t w[4]; };

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32 x 32 -> 64 bit multiplication per product (halves of it as two instructions cost twice as much)
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0, p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t hi0 = static_cast<uint32_t>(p0 >> 32), lo0 = static_cast<uint32_t>(p0);
    const uint32_t hi1 = static_cast<uint32_t>(p1 >> 32), lo1 = static_cast<uint32_t>(p1);
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  Words4 o; o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
  return o;
}

// The key of the per-coordinate random streams: which worker, which round, which stream.
struct RandKey {
  uint32_t worker, round_lo, round_hi_stream, seed_lo, seed_hi;
};

__device__ __forceinline__ RandKey make_rand_key(uint64_t seed, uint32_t worker, uint64_t round, uint32_t stream) {
  RandKey k;
  k.worker = worker; k.round_lo = static_cast<uint32_t>(round);
  k.round_hi_stream = static_cast<uint32_t>(round >> 32) | (stream << 30);
  k.seed_lo = static_cast<uint32_t>(seed); k.seed_hi = static_cast<uint32_t>(seed >> 32);
  return k;
}

// random word of coordinate i: output (i mod 4) of the block with counter (i / 4, worker, round...)
__device__ __forceinline__ uint32_t rand_word(const RandKey& k, uint32_t i) {
  const Words4 o = philox4x32_10(i >> 2, k.worker, k.round_lo, k.round_hi_stream, k.seed_lo, k.seed_hi);
  const uint32_t j = i & 3u;
  return j == 0 ? o.w[0] : j == 1 ? o.w[1] : j == 2 ? o.w[2] : o.w[3];
}

// random words of the four consecutive coordinates i0 .. i0+3 (one Philox block when i0 is a multiple of 4)
__device__ __forceinline__ Words4 rand_words4(const RandKey& k, uint32_t i0) {
  const Words4 a = philox4x32_10(i0 >> 2, k.worker, k.round_lo, k.round_hi_stream, k.seed_lo, k.seed_hi);
  const uint32_t sh = i0 & 3u;
  if (sh == 0) return a;
  const Words4 b = philox4x32_10((i0 >> 2) + 1u, k.worker, k.round_lo, k.round_hi_stream, k.seed_lo, k.seed_hi);
  Words4 o;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t j = sh + c;   // 1..6
    o.w[c] = j == 1 ? a.w[1] : j == 2 ? a.w[2] : j == 3 ? a.w[3] : j == 4 ? b.w[0] : j == 5 ? b.w[1] : b.w[2];
  }
  return o;
}

// `width` (<= 32) bits at bit offset `bit` of a little-endian stream of 32-bit words; words[n_words-1] is the last
__device__ __forceinline__ uint32_t get_bits(const uint32_t* words, uint64_t bit, uint32_t width) {
  if (width == 0) return 0;
  const uint64_t w = bit >> 5;
  const uint32_t sh = static_cast<uint32_t>(bit & 31);
  uint64_t v = words[w];
  if (sh + width > 32) v |= static_cast<uint64_t>(words[w + 1]) << 32;
  v >>= sh;
  return width == 32 ? static_cast<uint32_t>(v) : static_cast<uint32_t>(v) & ((1u << width) - 1u);
}

}  // namespace qsl
