// qsl_stream.h -- The kernels in front of the selection: unit-state initialisation, the sampled guess for Top_k
// (k_sample, k_sample_scan) and the one pass over HBM (k_stream: v = m + Delta, candidates to slots).
// Part of the single translation unit qsl.hip (included there, in this order: device, layout, select,
// encode, stream, lean, dense, decode); not a public header.
#pragma once

#include "qsl_device.h"
#include "qsl_layout.h"
#include "qsl_select.h"
#include "qsl_encode.h"

namespace {

// ------------------------------------------------------------------------------------------------
// one-time initialisation of the static part of the unit states (at qsl_create)
// ------------------------------------------------------------------------------------------------
__global__ void k_init(DevCtx c, uint32_t U) {
  const uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= U) return;
  const SegInfo& sg = c.segs[u % c.L];
  UnitState s = {};
  s.path = sg.mode; s.T = sg.mode == PATH_FAST ? sg.T_static : 0xFFFFFFFFu;
  // Rand_k: the keys are uniform words, the guess and the bins are fixed: 4096 bins over [T, 2^32)
  s.sh = 0;
  while (s.sh < 20 && ((0xFFFFFFFFu - s.T) >> s.sh) >= HBINS) ++s.sh;
  s.T_next = s.T; s.sh_next = s.sh; s.T_used = s.T;
  s.k_rem1 = sg.k; s.k_rem2 = sg.k;
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
__global__ __launch_bounds__(BIG) void k_sample(DevCtx c, const float* m, const float* delta, const float* xm, uint32_t R) {
  __shared__ uint32_t lh[HBINS];
  const SelInfo si = c.samps[blockIdx.x / R];            // one-dimensional grid, workers innermost, largest samples first
  const uint32_t seg = si.seg, w = blockIdx.x % R;
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
  // The blocks of a unit spread their counts over the unit's three histograms (the two of the later
  // digits are idle and zero now): 128 blocks adding into the same ~200 words queue up behind each other
  // (measured 10 us for one copy, 4 us for four); k_sample_scan adds the copies and clears them.
  flush_hist(lh, c.hist + ((static_cast<uint64_t>(w) * c.L + seg) * 3 + si.j % 3) * HBINS);
}

__global__ __launch_bounds__(BIG) void k_sample_scan(DevCtx c) {
  __shared__ uint64_t scratch[17];
  __shared__ uint32_t result[6];
  const uint32_t seg = c.fast_segs[blockIdx.x], w = blockIdx.y;
  const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
  const SegInfo& sg = c.segs[seg];
  // two ranks of the sample: r_s, far enough down for the guess to lie below the true threshold, and r_tau <= r_s,
  // about where the threshold itself lies -- the distance between the two sets the width of the candidates' bins
  find2_from_top<BIG, 3>(c.hist + u * 3 * HBINS, sg.r_tau, sg.r_s, scratch, result, true);
  if (threadIdx.x == 0) {
    const uint32_t bin_tau = result[0], bin_s = result[2];
    uint32_t sh = 11;                                   // 4096 bins over 8 x (estimated threshold - guess)
    while (sh < 20 && (1u << (sh - 11)) < bin_tau + 1 - bin_s) ++sh;
    c.units[u].T = bin_s << 20;                         // the guess: lower edge of the bin
    c.units[u].sh = sh;
  }
}

// ------------------------------------------------------------------------------------------------
// A unit of at most 4096 coordinates that has a k_stream block to itself (four waves, a chunk each): the block
// has the unit's values in registers when it has streamed them, so it goes on to select, order, norm and encode the
// unit itself -- radix digits of the k-th largest key in LDS, ranks by ballots and one exchange of the waves'
// counts -- while the other blocks of the launch keep streaming.  Lane l of the wave with chunk c holds the
// coordinates c * 1024 + t * 256 + l * 4 + j (t, j = 0..3) in v[t][j]; `cb` is the wave's first coordinate inside
// the unit (>= the unit's size for a wave without a chunk).
// ------------------------------------------------------------------------------------------------
template <int LEVEL>
__device__ __forceinline__ void stream_unit_hist(const uint32_t (&key)[16], uint32_t inside, uint32_t prefix, uint32_t* lh) {
#pragma unroll
  for (uint32_t i = 0; i < 16; ++i) {
    uint32_t bin;
    if (((inside >> i) & 1u) && level_bin<LEVEL>(key[i], prefix, &bin)) atomicAdd(&lh[bin], 1u);
  }
}

template <int SPARS>
__device__ void stream_block_unit(const DevCtx& c, const SegInfo& sg, uint64_t u, uint32_t w, uint64_t cb, const f4u (&v)[4],
                                  uint32_t worker0, uint64_t round, float* m_out, uint32_t* dbg_idx, uint16_t* dbg_level,
                                  uint32_t* lh, uint64_t* acc, uint64_t* scratch, uint32_t* result, uint32_t* s_wt,
                                  float* s_scale, uint32_t* s_count) {
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  uint32_t key[16], inside = 0;
#pragma unroll
  for (uint32_t t = 0; t < 4; ++t) {
    const uint64_t e = cb + t * 256 + lane * 4;
    Words4 rw = {{0u, 0u, 0u, 0u}};
    if (SPARS == QSL_RANDK && e < sg.size) rw = rand_words4(rk, static_cast<uint32_t>(sg.start + e));
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
      key[t * 4 + j] = SPARS == QSL_TOPK ? key_of_value(__float_as_uint(v[t][j])) : rw.w[j];
      inside |= (e + j < sg.size ? 1u : 0u) << (t * 4 + j);
    }
  }
  for (uint32_t i = threadIdx.x; i < HBINS; i += BLOCK) lh[i] = 0;
  for (uint32_t i = threadIdx.x; i < ACC_ROWS * acc_stride(c.quantizer); i += BLOCK) acc[i] = 0;
  __syncthreads();
  // the three digits of the k-th largest key -- unless the unit keeps every coordinate (a tensor of at most k
  // coordinates under a rule like k_t = min(d_t, 1000), Section 5.1.1): then there is nothing to find
  const bool all = sg.k == sg.size;                 // uniform over the block
  uint32_t tau = 0, need = 0;
  if (!all) {
    uint32_t above;
    stream_unit_hist<0>(key, inside, 0, lh);
    __syncthreads();
    uint32_t bin = find_from_top<BLOCK>(lh, sg.k, &above, scratch, result, true);
    uint32_t prefix = bin << 20, k_rem = sg.k - above;
    stream_unit_hist<1>(key, inside, prefix, lh);
    __syncthreads();
    bin = find_from_top<BLOCK>(lh, k_rem, &above, scratch, result, true);
    prefix |= bin << 8; k_rem -= above;
    stream_unit_hist<2>(key, inside, prefix, lh);
    __syncthreads();
    bin = find_from_top<BLOCK, 256>(lh, k_rem, &above, scratch, result, false);
    tau = prefix | bin; need = k_rem - above;
  }
  // ranks in coordinate order: wave (= chunk), then t, then lane, then j.  Counts packed as (#equal << 16 | #greater).
  uint32_t gm = 0, qm = 0;
#pragma unroll
  for (uint32_t i = 0; i < 16; ++i) {
    const bool in = (inside >> i) & 1u;
    gm |= (in && (all || key[i] > tau) ? 1u : 0u) << i;
    qm |= (in && !all && key[i] == tau ? 1u : 0u) << i;
  }
  uint32_t pre[4];
#pragma unroll
  for (uint32_t t = 0; t < 4; ++t) {
    uint32_t tot;
    pre[t] = wave_exclusive_scan32(__popc((gm >> (t * 4)) & 0xFu) | (__popc((qm >> (t * 4)) & 0xFu) << 16), &tot);
    if (lane == 0) s_wt[wave * 4 + t] = tot;
  }
  __syncthreads();
  uint32_t* oi = c.sel_idx + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint32_t* ov = c.sel_val + static_cast<uint64_t>(w) * c.K + sg.koff;
  uint64_t* mine = acc + (wave * 8 + (lane & 7u)) * acc_stride(c.quantizer);
  const uint32_t power = norm_power(c.quantizer);
  uint32_t base = 0;                                // counts of everything before (wave, t = 0)
  for (uint32_t i = 0; i < wave * 4; ++i) base += s_wt[i];
#pragma unroll
  for (uint32_t t = 0; t < 4; ++t) {
    const uint32_t mine_t = base + pre[t];
    uint32_t my_gt = mine_t & 0xFFFFu, my_eq = mine_t >> 16;
    const uint32_t gn = (gm >> (t * 4)) & 0xFu, qn = (qm >> (t * 4)) & 0xFu;
    if (gn | qn) {
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) {
        const bool is_gt = (gn >> j) & 1u, is_eq = (qn >> j) & 1u;
        if (is_gt || (is_eq && my_eq < need)) {
          const uint32_t pos = my_gt + min(my_eq, need);
          const uint32_t bits = __float_as_uint(v[t][j]);
          if (pos < sg.k) {
            oi[pos] = static_cast<uint32_t>(sg.start + cb + t * 256 + lane * 4 + j); ov[pos] = bits;
            add_digits(mine, bits, power);
          }
        }
        my_gt += is_gt; my_eq += is_eq;
      }
    }
    base += s_wt[wave * 4 + t];
  }
  if (threadIdx.x == 0) { c.units[u].cand = 0; c.units[u].fell_back = 0; }
  block_encode_tail<BLOCK, ACC_ROWS>(c, sg, w, u, tau, need, worker0, round, m_out, dbg_idx, dbg_level, acc, s_scale, s_count);
}

// ------------------------------------------------------------------------------------------------
// the streaming pass.  One wave per chunk of 1024 coordinates: 8 + 4 dwordx4 accesses with
// streaming (non-temporal) cache hints, then the chunk's candidates go to the chunk's slot.
//
// Slot of a chunk: lpc * 2 elements of 8 bytes (lpc = 4, 8, 16 or 32: 64 to 512 bytes).  Element 0 is the header (count, overflow offset);
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
                                                  uint32_t R, uint32_t* msg_zero, uint32_t* dbg_idx, uint16_t* dbg_level) {
  __shared__ uint2 s_stage[BLOCK / 64][64];
  // only for the units that a block of this kernel selects and encodes itself (segmented contexts)
  __shared__ uint32_t s_lh[SINGLE ? 1 : HBINS];
  __shared__ uint64_t s_acc[SINGLE ? 1 : ACC_ROWS * (ACC_SLOTS + 1)];
  __shared__ uint64_t s_scratch[17];
  __shared__ uint32_t s_result[2], s_wt[16], s_count;
  __shared__ float s_scale;
  __shared__ uint32_t s_stage_key[SPARS == QSL_RANDK ? BLOCK / 64 : 1][64];
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
  bool inblock = false;
  uint64_t first = static_cast<uint64_t>(wt) * CHUNK;                 // of the chunk, within the row
  uint32_t valid = static_cast<uint32_t>(min(static_cast<uint64_t>(CHUNK), one.size - first));
  if (!SINGLE) {
    const WtInfo wi = c.wts[wt];
    const SegInfo& s = c.segs[wi.seg];
    seg = wi.seg; chunk = wi.chunk; inblock = wi.inblock != 0; first = wi.first; valid = wi.valid;
    sg.start = s.start; sg.size = s.size; sg.slot_off = s.slot_off; sg.ovf_off = s.ovf_off;
    sg.lpc = s.lpc; sg.ovf_cap = s.ovf_cap;
  }
  const uint64_t u = static_cast<uint64_t>(w) * c.L + seg;
  const uint32_t T = c.units[u].T;
  const uint32_t path = c.units[u].path;
  const uint64_t row = static_cast<uint64_t>(w) * c.d + first;
  const float* mp = m + row;
  const float* dp = delta + row;
  const float* xp = DIFF ? xm + first : nullptr;
  float* op = m_out + row;
  f4u v[4];
  if (valid == CHUNK) {
    f4u a[4], b[4], x[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint32_t e = t * 256 + lane * 4;
      a[t] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(mp + e));
      b[t] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(dp + e));
      if (DIFF) x[t] = *reinterpret_cast<const f4u*>(xp + e);        // cached: the other workers read it too
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (DIFF) b[t] = x[t] - b[t];
      v[t] = a[t] + b[t];
      __builtin_nontemporal_store(v[t], reinterpret_cast<f4u*>(op + t * 256 + lane * 4));
    }
  } else {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t e = t * 256 + lane * 4 + j;
        float x = 0.0f;                                               // past the end: never a candidate
        if (e < valid) {
          const float dl = DIFF ? xp[e] - dp[e] : dp[e];
          x = mp[e] + dl; op[e] = x;
        }
        v[t][j] = x;
      }
    }
  }
  // segment-local; a wave that only fills up the block of a small unit has no chunk: nothing of it lies inside the unit
  const uint64_t cb = first - sg.start;
  bool nonfinite = false;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) nonfinite |= (__float_as_uint(v[t][j]) & 0x7FFFFFFFu) >= 0x7F800000u;
  }
  if (__ballot(nonfinite) != 0 && lane == 0) atomicOr(c.status, 1u);
  // `msg_zero` (the messages, if k_pack_sent is to put them together: it adds its fields to words that are zero): wave
  // wt clears the words wt * 64 .. wt * 64 + 63 of its worker's message (and on, a grid's width apart, if the message
  // is longer than that).  Here, behind the streaming accesses: ahead of them it cost the pass 1 %.
  if (msg_zero != nullptr && wt < (c.cap_words + 63u) / 64u)
    for (uint64_t q = static_cast<uint64_t>(wt) * 64 + lane; q < c.cap_words; q += static_cast<uint64_t>(c.NWT) * 64)
      msg_zero[static_cast<uint64_t>(w) * c.cap_words + q] = 0;
  if (!SINGLE && inblock) {                       // uniform over the block: it selects and encodes its unit itself
    const SegInfo unit = c.segs[seg];
    stream_block_unit<SPARS>(c, unit, u, w, cb, v, worker0, round, m_out, dbg_idx, dbg_level, s_lh, s_acc, s_scratch,
                             s_result, s_wt, &s_scale, &s_count);
    return;
  }
  if (path != PATH_FAST) return;                  // uniform over the wave: only a guessing unit collects candidates

  const RandKey rk = make_rand_key(c.seed, worker0 + w, round, 0);
  uint32_t pm = 0;                                                    // bit t*4+j: coordinate (t, j) is a candidate
  Words4 rws[4];                                                      // Rand_k: the keys, kept for the slot's key line
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    Words4 rw;
    if (SPARS == QSL_RANDK) { rw = rand_words4(rk, static_cast<uint32_t>(first + t * 256 + lane * 4)); rws[t] = rw; }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t key = SPARS == QSL_TOPK ? key_of_value(__float_as_uint(v[t][j])) : rw.w[j];
      const bool inside = static_cast<uint32_t>(t * 256 + lane * 4 + j) < valid;
      pm |= (inside && key >= T ? 1u : 0u) << (t * 4 + j);
    }
  }

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
            dst[pos++] = make_uint2(static_cast<uint32_t>(first + t * 256 + lane * 4 + j), __float_as_uint(v[t][j]));
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

}  // namespace
