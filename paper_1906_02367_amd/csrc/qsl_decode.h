// qsl_decode.h -- Reading messages: the stand-alone error update (k_add_rows, k_subtract_msg) and the master's
// aggregation (k_fill_zero, k_msg_directory, k_aggregate, k_aggregate_entries, k_aggregate_ranges,
// k_aggregate_dense_ranges, k_aggregate_dense), k_read_nnz.
// Part of the single translation unit qsl.hip (included there, in this order: device, layout, select,
// encode, stream, lean, dense, decode); not a public header.
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
  const bool counts = is_qsgd(c.quantizer) && c.L > 1 && !c.dense;
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L) + (counts ? c.L : 0);
  v.idx_bit0 = hdr * 32;
  v.code_bit0 = (hdr + (static_cast<uint64_t>(v.nnz) * c.w_idx + 31) / 32) * 32;
  return v;
}
__device__ __forceinline__ uint32_t msg_index(const DevCtx& c, const MsgView& v, uint32_t j) {
  if (c.dense) return j;                                 // the index-free format: entry j is coordinate j
  return get_bits(v.words, v.idx_bit0 + static_cast<uint64_t>(j) * c.w_idx, c.w_idx);
}
// the value a code field stands for, given the scale its segment transmitted
__device__ __forceinline__ float value_of_code(const DevCtx& c, uint32_t code, float scale) {
  if (is_qsgd(c.quantizer)) {
    // with indices only the levels 1..s are transmitted, as level - 1; the index-free format writes 0..s as they are
    const uint32_t level = (code & ((1u << c.w_lev) - 1u)) + (c.dense ? 0u : 1u);
    if (level == 0) return 0.0f;
    return qsgd_value(scale, level, c.s, (code >> c.w_lev) & 1u);
  }
  if (c.quantizer == QSL_FP32) return __uint_as_float(code);
  return code ? -scale : scale;
}
__device__ __forceinline__ float msg_value(const DevCtx& c, const MsgView& v, uint32_t j, uint32_t idx) {
  const uint32_t code = get_bits(v.words, v.code_bit0 + static_cast<uint64_t>(j) * c.w_val, c.w_val);
  const uint32_t seg = c.L == 1 ? 0u : seg_of_coord(c, idx);
  return value_of_code(c, code, __uint_as_float(v.words[1 + seg]));
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
constexpr uint32_t AGG_DIR_MIN = 4096;   // messages expected to be at least this long are searched through their directories
// k_aggregate_ranges takes over from 24 listed messages on when they are long, from 56 on in any case (measured, 8 workers'
// messages repeated: 99,400 entries each: 15 / 32 / 64 messages 138 / 442 / 1480 us by look-ups, 170 / 277 / 473 us by
// ranges; ~1,600 entries each: 14 / 31 / 105 us against 44 / 64 / 93 us)
constexpr uint32_t AGG_RANGES_MIN_R_LONG = 24, AGG_RANGES_MIN_R = 56;

// Directory of a long message: dir[t] = number of entries whose coordinate lies below t * 1024, for
// t = 0 .. ndir - 1 (ndir = ceil(d / 1024) + 1, so dir[ndir - 1] = nnz).  Entry j fills the slots between
// its predecessor's 1024-block and its own; the last entry also fills the rest.  A lookup then needs
// dir[t], dir[t + 1] and a binary search over the few entries of one 1024-block instead of log2(nnz)
// dependent probes of the whole message.
__global__ __launch_bounds__(BLOCK) void k_msg_directory(DevCtx c, const uint8_t* msg, RowList rows, uint32_t* dir,
                                                         uint32_t ndir, uint32_t* dense_list) {
  const uint32_t q = blockIdx.y;
  const MsgView v = view_msg(c, msg, rows.row[q]);
  uint32_t* mine = dir + static_cast<uint64_t>(q) * ndir;
  if (dense_list && q == 0 && blockIdx.x == 0 && threadIdx.x == 0) dense_list[0] = 0;    // the list k_aggregate_ranges fills
  const uint32_t nth = gridDim.x * BLOCK, tid = blockIdx.x * BLOCK + threadIdx.x;
  if (v.nnz == 0) { for (uint32_t t = tid; t < ndir; t += nth) mine[t] = 0; return; }
  for (uint32_t j = tid; j < v.nnz; j += nth) {
    const uint32_t cur = min(msg_index(c, v, j) >> AGG_DIR_SHIFT, ndir - 2);           // clamp: a malformed index
    const uint32_t first = j ? min(msg_index(c, v, j - 1) >> AGG_DIR_SHIFT, ndir - 2) + 1 : 0u;
    for (uint32_t t = first; t <= cur; ++t) mine[t] = j;                // empty when the predecessor shares the block
    if (j == v.nnz - 1) for (uint32_t t = cur + 1; t < ndir; ++t) mine[t] = v.nnz;
  }
}

// Short messages (no directory).  Entry j of the q-th listed message is served by 8 threads, which look its
// coordinate up in the other listed messages (binary search on the packed, ascending indices).  The coordinate is
// written by the earliest listed message that holds it -- one writer per coordinate, no atomics --
// and the values are added in list order, so the result does not depend on the schedule.
__global__ __launch_bounds__(BLOCK) void k_aggregate(DevCtx c, const uint8_t* msg, RowList rows, uint32_t R,
                                                     float scale, int accumulate, float* out) {
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
        const int64_t pos = msg_find(c, other, idx);
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

// Long messages (with directories).  One thread per entry: the thread that holds entry j of the q-th listed
// message looks its coordinate up in the other listed messages itself, AGG_GROUP messages at a time with the
// binary searches advancing in step (their probes are independent loads, so a step costs one memory round trip,
// not one per message); a directory narrows every search to the entries of one 1024-block.  The rule is the same -- the
// earliest listed message that holds a coordinate writes it, the values are added in list order -- but a wave
// serves 64 entries instead of 8, and kernels of this kind are bound by the number of waves they start
// (8 messages of 99,400 entries: 104 us with 8 threads per entry, 55 us this way; short messages are the
// other way round: 8 x 543 entries 8 us against 16 us).  Four searches at a time: with eight the kernel needs 83
// registers (5 waves per SIMD) and takes 56.6 us on those messages, with four 51 registers and 53 us, with two 58 us.
constexpr uint32_t AGG_GROUP = 4;

struct GroupSearch {
  MsgView v[AGG_GROUP];
  uint32_t lo[AGG_GROUP], hi[AGG_GROUP];
  int64_t pos[AGG_GROUP];       // where the coordinate is in message g, or -1
};

// positions of coordinate idx in n (<= 8) of the other listed messages: the o-th other message, o = o0 .. o0 + n - 1,
// is list entry o for o < q and o + 1 from there on.  The loads of a step are unconditional (a closed search
// reads entry 0 again, which every message buffer has room for) so that all of a group are in flight together.
// `fixed_pos` >= 0: where the coordinate stands in every message that holds all K entries (a segment kept whole under a
// quantiser that drops nothing: its entries are at the same places in every such message) -- no search then.
__device__ __forceinline__ void group_find(const DevCtx& c, const uint8_t* msg, const RowList& rows, uint32_t o0, uint32_t n,
                                           uint32_t q, uint32_t idx, const uint32_t* dir, uint32_t ndir, int64_t fixed_pos,
                                           GroupSearch& s) {
  const uint32_t t = idx >> AGG_DIR_SHIFT;
  uint32_t nnz[AGG_GROUP], dlo[AGG_GROUP], dhi[AGG_GROUP];
#pragma unroll
  for (uint32_t g = 0; g < AGG_GROUP; ++g) {                // headers and directory cells: one batch of loads
    const uint32_t o = min(o0 + g, o0 + n - 1);             // slots beyond n repeat the last message and stay closed
    const uint32_t p = o + (o >= q ? 1u : 0u);
    s.v[g].words = reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(rows.row[p]) * c.cap_words * 4);
    nnz[g] = s.v[g].words[0];
    dlo[g] = dir ? dir[static_cast<uint64_t>(p) * ndir + t] : 0u;
    dhi[g] = dir ? dir[static_cast<uint64_t>(p) * ndir + t + 1] : 0xFFFFFFFFu;
  }
  const bool counts = is_qsgd(c.quantizer) && c.L > 1;
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L) + (counts ? c.L : 0);
#pragma unroll
  for (uint32_t g = 0; g < AGG_GROUP; ++g) {
    s.v[g].nnz = min(nnz[g], c.K);
    s.v[g].idx_bit0 = hdr * 32;
    s.v[g].code_bit0 = (hdr + (static_cast<uint64_t>(s.v[g].nnz) * c.w_idx + 31) / 32) * 32;
    s.pos[g] = -1; s.lo[g] = 0; s.hi[g] = 0;
    if (g < n) {
      if (s.v[g].nnz == c.d) s.pos[g] = idx;               // every coordinate is there (k = d): entry j is coordinate j
      else if (fixed_pos >= 0 && s.v[g].nnz == c.K) s.pos[g] = fixed_pos;
      else { s.hi[g] = min(dhi[g], s.v[g].nnz); s.lo[g] = min(dlo[g], s.hi[g]); }
    }
  }
  for (uint32_t step = 0; step < 33; ++step) {             // a window of 2^32 entries is empty after 33 halvings
    bool open = false;
    uint32_t mid[AGG_GROUP], w0[AGG_GROUP], w1[AGG_GROUP];
#pragma unroll
    for (uint32_t g = 0; g < AGG_GROUP; ++g) {
      const bool active = s.lo[g] < s.hi[g];
      open = open || active;
      mid[g] = active ? s.lo[g] + ((s.hi[g] - s.lo[g]) >> 1) : 0u;
      const uint64_t bit = s.v[g].idx_bit0 + static_cast<uint64_t>(mid[g]) * c.w_idx;
      w0[g] = s.v[g].words[bit >> 5];
      w1[g] = s.v[g].words[(bit >> 5) + 1];
    }
    if (!open) break;
#pragma unroll
    for (uint32_t g = 0; g < AGG_GROUP; ++g) {
      const uint64_t bit = s.v[g].idx_bit0 + static_cast<uint64_t>(mid[g]) * c.w_idx;
      const uint32_t x = static_cast<uint32_t>(((static_cast<uint64_t>(w1[g]) << 32) | w0[g]) >> (bit & 31)) &
                         (c.w_idx == 32 ? 0xFFFFFFFFu : (1u << c.w_idx) - 1u);
      if (s.lo[g] < s.hi[g]) {
        if (x == idx) { s.pos[g] = mid[g]; s.hi[g] = s.lo[g]; }
        else if (x < idx) s.lo[g] = mid[g] + 1;
        else s.hi[g] = mid[g];
      }
    }
  }
}

__global__ __launch_bounds__(BLOCK) void k_aggregate_entries(DevCtx c, const uint8_t* msg, RowList rows, uint32_t R,
                                                             float scale, int accumulate, float* out, const uint32_t* dir,
                                                             uint32_t ndir) {
  const uint32_t q = blockIdx.y;
  const MsgView mine = view_msg(c, msg, rows.row[q]);
  const uint32_t stride = gridDim.x * BLOCK;
  GroupSearch s;
  for (uint32_t j = blockIdx.x * BLOCK + threadIdx.x; j < mine.nnz; j += stride) {
    const uint32_t idx = msg_index(c, mine, j);
    if (idx >= c.d) { atomicOr(c.status, 4u); continue; }          // malformed message
    const uint32_t seg = c.L == 1 ? 0u : seg_of_coord(c, idx);
    // a segment that is kept whole (k = size, e.g. the small tensors under a per-tensor rule) by a quantiser that drops
    // nothing stands at the same places in every full message
    int64_t fixed_pos = -1;
    if (c.L > 1 && !is_qsgd(c.quantizer) && mine.nnz == c.K && c.seg_whole[seg])
      fixed_pos = static_cast<int64_t>(c.seg_koff[seg]) + (idx - c.seg_start[seg]);
    // ... so if the first listed message is full it owns the coordinate: nothing to look up for the others' threads
    if (fixed_pos >= 0 && q > 0 &&
        reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(rows.row[0]) * c.cap_words * 4)[0] == c.K) continue;
    const uint32_t my_code = get_bits(mine.words, mine.code_bit0 + static_cast<uint64_t>(j) * c.w_val, c.w_val);
    float acc = value_of_code(c, my_code, __uint_as_float(mine.words[1 + seg]));
    bool owned = false;                                            // an earlier listed message holds the coordinate: its thread writes it
    for (uint32_t o0 = 0; o0 + 1 < R && !owned; o0 += AGG_GROUP) {
      const uint32_t n = min(AGG_GROUP, R - 1 - o0);
      group_find(c, msg, rows, o0, n, q, idx, dir, ndir, fixed_pos, s);
      uint32_t w0[AGG_GROUP], w1[AGG_GROUP]; float sc[AGG_GROUP];
#pragma unroll
      for (uint32_t g = 0; g < AGG_GROUP; ++g) {              // code fields and scales of the group, found or not: one batch
        const uint64_t bit = s.v[g].code_bit0 + static_cast<uint64_t>(s.pos[g] >= 0 ? s.pos[g] : 0) * c.w_val;
        const uint64_t w = min(bit >> 5, static_cast<uint64_t>(c.cap_words) - 2);
        w0[g] = s.v[g].words[w]; w1[g] = s.v[g].words[w + 1];
        sc[g] = __uint_as_float(s.v[g].words[1 + seg]);
        if (s.pos[g] >= 0 && o0 + g < q) owned = true;
      }
#pragma unroll
      for (uint32_t g = 0; g < AGG_GROUP; ++g) {
        if (s.pos[g] >= 0 && o0 + g >= q) {
          const uint64_t bit = s.v[g].code_bit0 + static_cast<uint64_t>(s.pos[g]) * c.w_val;
          const uint64_t w = min(bit >> 5, static_cast<uint64_t>(c.cap_words) - 2);        // the pair of words that was loaded
          const uint32_t code = static_cast<uint32_t>(((static_cast<uint64_t>(w1[g]) << 32) | w0[g]) >> (bit - w * 32)) &
                                (c.w_val == 32 ? 0xFFFFFFFFu : (1u << c.w_val) - 1u);
          acc = acc + value_of_code(c, code, sc[g]);
        }
      }
    }
    if (owned) continue;
    const float term = scale * acc;
    out[idx] = accumulate ? out[idx] + term : term;
  }
}

// Many messages: work linear in the number of entries.  A wave owns 1024 consecutive coordinates (one cell of the
// directories): lane p knows where listed message p's entries of that range begin and end; the entries of as many
// messages as the staging list holds are decoded side by side into LDS, then added into an LDS image of the range
// message after message, in list order -- the entries of one message have distinct coordinates, so the additions of
// one message do not meet, and the order of the fp32 additions is that of k_aggregate.  No look-ups in other
// messages: the cost of the kernels above grows with the square of the number of messages (8, 15, 32, 64 messages
// of 99,400 entries: 55, 138, 442, 1480 us), this one's with their number.  A range that holds more than 4096
// entries in all (segments kept whole: every message has every coordinate) would keep one wave busy for long, so
// the waves only list such ranges and a second launch gives each of them a block of 1024 threads.
constexpr uint32_t AGG_RANGE = 1u << AGG_DIR_SHIFT;      // coordinates per range
constexpr uint32_t AGG_DENSE_MIN = 4096;                 // entries in a range from which a whole block takes it
constexpr uint32_t AGG_DENSE_BLOCKS = 512;

template <uint32_t NT>
__device__ __forceinline__ void range_barrier() {
  if (NT == WAVE) {                                      // one wave, lanes in lockstep: order the LDS traffic only
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  } else __syncthreads();
}

// One range by NT threads (NT = 64: a wave; else a block).  STAGE: entries the staging list holds (>= 1024, so that one
// message's share of a range fits).  Returns false, having done nothing, if LIST and the range holds AGG_DENSE_MIN
// entries or more (uniform over the threads).
template <uint32_t NT, uint32_t STAGE, bool LIST>
__device__ bool aggregate_range(const DevCtx& c, const uint8_t* msg, const RowList& rows, uint32_t R, float scale, int accumulate,
                                float* out, const uint32_t* dir, uint32_t ndir, uint32_t t, float* s_acc, uint8_t* s_has,
                                uint32_t* s_loc, float* s_val) {
  const uint32_t lane = lane_id(), tid = threadIdx.x;
  const uint64_t base = static_cast<uint64_t>(t) << AGG_DIR_SHIFT;
  // lane p (of every wave): listed message p -- its row, its length, its entries [lo, hi) that fall into this range
  uint32_t my_row = 0, my_nnz = 0, lo = 0, hi = 0;
  if (lane < R) {
    my_row = rows.row[lane];
    my_nnz = min(reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(my_row) * c.cap_words * 4)[0], c.K);
    lo = min(dir[static_cast<uint64_t>(lane) * ndir + t], my_nnz);
    hi = min(dir[static_cast<uint64_t>(lane) * ndir + t + 1], my_nnz);
    if (hi < lo) hi = lo;
    if (hi - lo > AGG_RANGE) hi = lo + AGG_RANGE;        // a well-formed message has at most one entry per coordinate
  }
  const uint32_t cnt = hi - lo;
  if (__ballot(cnt != 0) == 0) return true;              // nothing to add here
  if (LIST && wave_sum(cnt) >= AGG_DENSE_MIN) return false;
  for (uint32_t i = tid; i < AGG_RANGE; i += NT) s_has[i] = 0;
  const bool counts = is_qsgd(c.quantizer) && c.L > 1;
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L) + (counts ? c.L : 0);
  const uint32_t idx_mask = c.w_idx == 32 ? 0xFFFFFFFFu : (1u << c.w_idx) - 1u;
  // the segments of the range's first and last coordinate: mostly the same one
  const uint32_t seg_lo = c.L == 1 ? 0u : seg_of_coord(c, static_cast<uint32_t>(base));
  const uint32_t seg_hi = c.L == 1 ? 0u : seg_of_coord(c, static_cast<uint32_t>(min<uint64_t>(base + AGG_RANGE, c.d) - 1));
  uint32_t p0 = 0;
  while (p0 < R) {                                       // uniform over the threads
    // the batch p0 .. p1 - 1: as many messages as the staging list holds (at least one)
    uint32_t tot;
    const uint32_t before = wave_exclusive_scan32(lane >= p0 && lane < R ? cnt : 0u, &tot);
    const uint64_t over = __ballot(lane > p0 && lane < R && before + cnt > STAGE);
    const uint32_t p1 = over ? static_cast<uint32_t>(__ffsll(static_cast<unsigned long long>(over)) - 1) : R;
    const uint32_t n_staged = p1 < R ? __shfl(before, p1, WAVE) : tot;
    const uint64_t in_batch = __ballot(cnt != 0 && lane >= p0 && lane < p1);
    // decode the batch side by side, 4 x NT staged entries per step with their loads in flight together: staged entry
    // f belongs to the last message x of the batch with before_x <= f
    constexpr uint32_t UN = 4;
    for (uint32_t f0 = 0; f0 < n_staged; f0 += UN * NT) {
      uint32_t q_row[UN], q_nnz[UN], q_lo[UN], q_before[UN];
#pragma unroll
      for (uint32_t u = 0; u < UN; ++u) { q_row[u] = 0; q_nnz[u] = 0; q_lo[u] = 0; q_before[u] = 0; }
      for (uint64_t left = in_batch; left; left &= left - 1) {      // the batch's messages that have entries here, in order
        const int x = __ffsll(static_cast<unsigned long long>(left)) - 1;     // (uniform: every lane takes part in the shuffles)
        const uint32_t bx = __shfl(before, x, WAVE);
        const uint32_t rx = __shfl(my_row, x, WAVE), nx = __shfl(my_nnz, x, WAVE), lx = __shfl(lo, x, WAVE);
#pragma unroll
        for (uint32_t u = 0; u < UN; ++u)
          if (f0 + u * NT + tid >= bx) { q_row[u] = rx; q_nnz[u] = nx; q_lo[u] = lx; q_before[u] = bx; }
      }
      uint32_t idx[UN], code[UN];
      const uint32_t* words[UN];
#pragma unroll
      for (uint32_t u = 0; u < UN; ++u) {
        const uint32_t f = f0 + u * NT + tid;
        words[u] = reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(q_row[u]) * c.cap_words * 4);
        idx[u] = 0xFFFFFFFFu; code[u] = 0;
        if (f < n_staged) {
          const uint32_t j = q_lo[u] + (f - q_before[u]);
          idx[u] = get_bits(words[u], hdr * 32 + static_cast<uint64_t>(j) * c.w_idx, c.w_idx) & idx_mask;
          const uint64_t code_bit0 = (hdr + (static_cast<uint64_t>(q_nnz[u]) * c.w_idx + 31) / 32) * 32;
          code[u] = get_bits(words[u], code_bit0 + static_cast<uint64_t>(j) * c.w_val, c.w_val);
        }
      }
#pragma unroll
      for (uint32_t u = 0; u < UN; ++u) {
        const uint32_t f = f0 + u * NT + tid;
        if (f < n_staged) {
          uint32_t loc = 0xFFFFFFFFu;
          float val = 0.0f;
          if (idx[u] >= base && idx[u] < base + AGG_RANGE && idx[u] < c.d) {
            const uint32_t seg = c.L == 1 ? 0u : seg_lo == seg_hi ? seg_lo : seg_of_coord(c, idx[u]);
            val = value_of_code(c, code[u], __uint_as_float(words[u][1 + seg]));
            loc = static_cast<uint32_t>(idx[u] - base);
          } else atomicOr(c.status, 4u);                   // malformed message: the entry is skipped
          s_loc[f] = loc; s_val[f] = val;
        }
      }
    }
    range_barrier<NT>();
    // add them message after message
    for (uint64_t left = in_batch; left; left &= left - 1) {
      const int x = __ffsll(static_cast<unsigned long long>(left)) - 1;
      const uint32_t bx = __shfl(before, x, WAVE), cx = __shfl(cnt, x, WAVE);
      for (uint32_t i = tid; i < cx; i += NT) {
        const uint32_t loc = s_loc[bx + i];
        if (loc != 0xFFFFFFFFu) {
          const float v = s_val[bx + i];
          s_acc[loc] = s_has[loc] ? s_acc[loc] + v : v;
          s_has[loc] = 1;
        }
      }
      range_barrier<NT>();
    }
    p0 = p1;
  }
  for (uint32_t i = tid; i < AGG_RANGE; i += NT) {
    if (s_has[i]) {
      const float term = scale * s_acc[i];
      out[base + i] = accumulate ? out[base + i] + term : term;
    }
  }
  return true;
}

// a wave per range; the ranges with too many entries for one wave go to `dense_list` (dense_list[0] counts them)
__global__ __launch_bounds__(64) void k_aggregate_ranges(DevCtx c, const uint8_t* msg, RowList rows, uint32_t R, float scale,
                                                         int accumulate, float* out, const uint32_t* dir, uint32_t ndir,
                                                         uint32_t* dense_list) {
  __shared__ float s_acc[AGG_RANGE];
  __shared__ uint8_t s_has[AGG_RANGE];
  __shared__ uint32_t s_loc[1024];
  __shared__ float s_val[1024];
  if (!aggregate_range<64, 1024, true>(c, msg, rows, R, scale, accumulate, out, dir, ndir, blockIdx.x, s_acc, s_has, s_loc, s_val) &&
      threadIdx.x == 0)
    dense_list[1 + atomicAdd(&dense_list[0], 1u)] = blockIdx.x;
}

// a block of 1024 threads per listed range
__global__ __launch_bounds__(1024) void k_aggregate_dense_ranges(DevCtx c, const uint8_t* msg, RowList rows, uint32_t R,
                                                                 float scale, int accumulate, float* out, const uint32_t* dir,
                                                                 uint32_t ndir, const uint32_t* dense_list) {
  __shared__ float s_acc[AGG_RANGE];
  __shared__ uint8_t s_has[AGG_RANGE];
  __shared__ uint32_t s_loc[8192];
  __shared__ float s_val[8192];
  const uint32_t n = min(dense_list[0], ndir - 1);
  for (uint32_t li = blockIdx.x; li < n; li += gridDim.x) {
    const uint32_t t = dense_list[1 + li];
    if (t < ndir - 1)
      aggregate_range<1024, 8192, false>(c, msg, rows, R, scale, accumulate, out, dir, ndir, t, s_acc, s_has, s_loc, s_val);
    __syncthreads();                                     // the LDS arrays are reused for the block's next range
  }
}

// The master line when every message holds every coordinate (an operator with k = d whose quantiser drops
// nothing, e.g. the sign of the whole vector): entry j of a message is coordinate j, so the sum is a plain
// pass over the coordinates, in the same list order and with the same roundings as k_aggregate.  An
// all-zero (empty) message adds nothing; any other entry count is reported as a malformed message.
// four consecutive coordinates from j0 on (nj of them exist); `o`: what `out` holds there (if accumulate)
__device__ __forceinline__ void aggregate_dense_quad(const DevCtx& c, const uint8_t* __restrict__ msg, const RowList& rows, uint32_t R,
                                                     float scale, int accumulate, float* __restrict__ out, uint64_t code_bit0,
                                                     uint64_t j0, uint32_t nj, f4u o) {
  uint32_t seg[4] = {0u, 0u, 0u, 0u};
  if (c.L > 1) {
    seg[0] = seg_of_coord(c, static_cast<uint32_t>(j0));
    seg[3] = seg_of_coord(c, static_cast<uint32_t>(j0 + nj - 1));
    seg[1] = seg[2] = seg[0];
    if (seg[3] != seg[0]) {
      seg[1] = nj > 1 ? seg_of_coord(c, static_cast<uint32_t>(j0 + 1)) : seg[0];
      seg[2] = nj > 2 ? seg_of_coord(c, static_cast<uint32_t>(j0 + 2)) : seg[0];
    }
  }
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  bool first = true;
  for (uint32_t p = 0; p < R; ++p) {
    const uint32_t* words = reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(rows.row[p]) * c.cap_words * 4);
    const uint32_t nnz = words[0];
    if (nnz != c.d) {
      if (nnz != 0 && j0 == 0) atomicOr(c.status, 4u);
      continue;
    }
    // the codes of the four coordinates are consecutive in the stream: up to 8 bits each come in one read
    // (77 -> 62 us for two messages of 25.6 M one-bit codes; issuing the reads of several messages together, or a
    // wave per 1024 coordinates as in the streaming pass, were both slower again: 72-77 us)
    const bool packed = c.w_val <= 8;                      // uniform
    const uint32_t four = packed ? get_bits(words, code_bit0 + j0 * c.w_val, nj * c.w_val) : 0u;
    const float scale0 = __uint_as_float(words[1 + seg[0]]);
#pragma unroll
    for (uint32_t jj = 0; jj < 4; ++jj) {
      if (jj < nj) {
        const uint32_t code = packed ? (four >> (jj * c.w_val)) & ((1u << c.w_val) - 1u)
                                     : get_bits(words, code_bit0 + (j0 + jj) * c.w_val, c.w_val);
        const float sc = seg[jj] == seg[0] ? scale0 : __uint_as_float(words[1 + seg[jj]]);
        const float val = value_of_code(c, code, sc);
        acc[jj] = first ? val : acc[jj] + val;
      }
    }
    first = false;
  }
  if (first && accumulate) return;                       // no message had anything to add
#pragma unroll
  for (uint32_t jj = 0; jj < 4; ++jj) {
    const float term = scale * acc[jj];
    o[jj] = first ? 0.0f : accumulate ? o[jj] + term : term;
  }
  if (nj == 4) *reinterpret_cast<f4u*>(out + j0) = o;
  else for (uint32_t jj = 0; jj < nj; ++jj) out[j0 + jj] = o[jj];
}

// A thread takes two groups of four consecutive coordinates at a time, a grid's width apart; what `out` holds of both is
// read first (one group: 62 us for two messages of 25.6 M one-bit codes; its read of `out` before those of the messages
// instead of after them: 59 us; two groups: 57 us; with streaming hints on `out`, which the next round's call finds
// partly in the last-level cache otherwise: 61 us).
__global__ __launch_bounds__(BLOCK) void k_aggregate_dense(DevCtx c, const uint8_t* __restrict__ msg, RowList rows, uint32_t R,
                                                           float scale, int accumulate, float* __restrict__ out) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * BLOCK;
  const uint64_t n4 = (c.d + 3) / 4;
  const bool counts = is_qsgd(c.quantizer) && c.L > 1 && !c.dense;
  const uint64_t hdr = 1 + static_cast<uint64_t>(c.L) + (counts ? c.L : 0);
  const uint64_t code_bit0 = (hdr + (c.d * c.w_idx + 31) / 32) * 32;      // of a message that holds all d entries
  for (uint64_t g = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x; g < n4; g += 2 * stride) {
    const uint64_t ja = g * 4, jb = (g + stride) * 4;
    const uint32_t na = static_cast<uint32_t>(min<uint64_t>(4, c.d - ja));
    const uint32_t nb = g + stride < n4 ? static_cast<uint32_t>(min<uint64_t>(4, c.d - jb)) : 0u;
    f4u oa = {0.f, 0.f, 0.f, 0.f}, ob = {0.f, 0.f, 0.f, 0.f};
    if (accumulate) {
      if (na == 4) oa = *reinterpret_cast<const f4u*>(out + ja);
      else for (uint32_t jj = 0; jj < na; ++jj) oa[jj] = out[ja + jj];
      if (nb == 4) ob = *reinterpret_cast<const f4u*>(out + jb);
      else for (uint32_t jj = 0; jj < nb; ++jj) ob[jj] = out[jb + jj];
    }
    aggregate_dense_quad(c, msg, rows, R, scale, accumulate, out, code_bit0, ja, na, oa);
    if (nb) aggregate_dense_quad(c, msg, rows, R, scale, accumulate, out, code_bit0, jb, nb, ob);
  }
}

__global__ void k_read_nnz(DevCtx c, const uint8_t* msg, uint32_t R, uint32_t* out) {
  const uint32_t r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < R) out[r] = reinterpret_cast<const uint32_t*>(msg + static_cast<uint64_t>(r) * c.cap_words * 4)[0];
}

}  // namespace
