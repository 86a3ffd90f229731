// qsl_decode.h -- Reading messages: the stand-alone error update (k_add_rows, k_subtract_msg) and the master's
// aggregation (k_fill_zero, k_msg_directory, k_aggregate), k_read_nnz.
// Part of the single translation unit qsl.hip (included there, in this order: layout, stream, select,
// encode, decode); not a public header.
#pragma once

#include "qsl_device.h"
#include "qsl_layout.h"

namespace {

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

// The master line when every message holds every coordinate (an operator with k = d whose quantiser drops
// nothing, e.g. the sign of the whole vector): entry j of a message is coordinate j, so the sum is a plain
// pass over the coordinates, in the same list order and with the same roundings as k_aggregate.  An
// all-zero (empty) message adds nothing; any other entry count is reported as a malformed message.
__global__ __launch_bounds__(BLOCK) void k_aggregate_dense(DevCtx c, const uint8_t* msg, RowList rows, uint32_t R,
                                                           float scale, int accumulate, float* out) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * BLOCK;
  for (uint64_t j = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x; j < c.d; j += stride) {
    float acc = 0.0f;
    bool first = true;
    for (uint32_t p = 0; p < R; ++p) {
      const MsgView v = view_msg(c, msg, rows.row[p]);
      if (v.nnz != c.d) {
        if (v.nnz != 0 && j == 0) atomicOr(c.status, 4u);
        continue;
      }
      const float val = msg_value(c, v, static_cast<uint32_t>(j), static_cast<uint32_t>(j));
      acc = first ? val : acc + val;
      first = false;
    }
    const float term = scale * acc;
    if (!first) out[j] = accumulate ? out[j] + term : term;
    else if (!accumulate) out[j] = 0.0f;
  }
}

__global__ void k_read_nnz(DevCtx c, const uint8_t* msg, uint32_t R, uint32_t* out) {
  const uint32_t r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < R) out[r] = reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(r) * c.cap_words * 4)[0];
}

}  // namespace
