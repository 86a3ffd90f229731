// qsl_layout.h -- Shared by all kernels of the library: tuning constants, the per-segment plan and per-unit state as they
// lie in device memory, and the histogram helpers of the radix selection.
// Part of the single translation unit qsl.hip (included there, in this order: device, layout, select,
// encode, stream, lean, dense, decode); not a public header.
#pragma once

#include "qsl_device.h"
#include "qsl.h"

using namespace qsl;

namespace {

constexpr uint32_t CHUNK = 1024;           // coordinates one wave streams: 4 x (64 lanes x 4)
constexpr uint32_t BLOCK = 256;
constexpr uint32_t HBINS = 4096;           // radix digits: 12 + 12 + 8 bits of the 32-bit rank key
constexpr uint32_t ACC_SLOTS = 40;         // 32-bit digits of the exact accumulator: fourth powers of fp32 values span 4 * 254 + 96 bits, plus 32 for their number
constexpr uint32_t MAX_SAMPLE_BLOCKS = 128; // blocks (of 1024 threads) per unit of the sampling kernel: 1 .. 128
constexpr uint32_t MAX_SELECT_BLOCKS = 64; // blocks (of 1024 threads) per unit of the selection kernels: 1 .. 64
constexpr uint32_t BIG = 1024;             // threads of the sampling and selection kernels
constexpr uint32_t MAX_QB_INLINE = 4096;   // above this many quantise blocks a separate prefix kernel runs
constexpr uint32_t NSUB = 64;              // candidate counters per unit: chunk t adds to counter t mod 64
constexpr uint32_t PAD = 64;               // words between two counters: atomics that share a cache line serialise
constexpr uint32_t CTR_OVF = NSUB;         // counter NSUB: cursor of the unit's overflow pool
constexpr uint32_t CTR_FAIL = NSUB + 1;    // counter NSUB + 1: set when the overflow pool ran out
constexpr uint32_t CTR_LIST = NSUB + 2;    // counter NSUB + 2: entries in the unit's list of threshold-bin candidates
constexpr uint32_t CTR_LINES = NSUB + 3;
constexpr uint32_t LISTCAP = 256;          // entries of that list; a threshold bin that holds more sends the unit to the block-wide selection

enum : uint32_t { PATH_FAST = 0, PATH_GENERAL = 1, PATH_FALLBACK = 2, PATH_SMALL = 3, PATH_FULL = 4 };
constexpr uint32_t MAX_FULL_BLOCKS = 512;  // blocks per unit of k_full (each ends with up to 20 atomics on the unit's digit counters)
constexpr uint32_t SMALL_CHUNKS = 4;       // a unit of at most 4 chunks (4096 coordinates) is always selected by one block
constexpr uint32_t BLOCK_PER = 40;         // coordinates a thread of the one-block selection holds at most ...
constexpr uint32_t BLOCK_MAX = BLOCK_PER * 1024;   // ... so a unit too dense to guess goes that way up to 40,960 coordinates

struct SegInfo {
  uint64_t start, size;
  uint64_t slot_off;     // first slot element (uint2) of this segment inside one worker's slot area
  uint64_t ovf_off;      // first entry of this segment inside one worker's overflow pool
  uint64_t d0_off;       // first entry of this segment inside one worker's dense candidate lists
  uint32_t k, koff;      // koff: first slot in the [K] selected arrays
  uint32_t nwt;          // chunks of 1024 coordinates
  uint32_t d0_cap;       // entries of the dense candidate list
  uint32_t wc_base;      // first per-wave counter of this segment (per worker)
  uint32_t cb_base, ncb; // compaction blocks: index of the first one (per worker), how many
  uint32_t nsamp;        // blocks of this unit in the sampling kernel
  uint32_t mode;         // PATH_FAST, PATH_GENERAL, PATH_SMALL or PATH_FULL, decided on the host from (size, k)
  uint32_t lpc;          // slot size: lpc * 16 bytes per chunk (4: 64 bytes, 8: one 128-byte line, 16: two lines, 32: four)
  uint32_t ovf_cap;      // entries of the overflow pool
  uint32_t n_runs;       // sample: runs of 64 consecutive coordinates
  uint32_t r_s;          // sample rank that defines the guess
  uint32_t T_static;     // Rand_k: analytic guess
  uint32_t nsel;         // blocks of this unit in the selection kernels
  uint32_t samp_stride;  // sample: distance between the starts of two runs (64: the whole unit is read)
  uint32_t r_warm;       // rank (among this call's candidates) whose bin edge becomes the next call's guess
  uint32_t r_tau;        // sample rank that estimates the threshold itself (for the width of the histogram bins)
  uint32_t fidx;         // number of this segment among the guessing ones
  uint32_t in_stream;    // 1: a block of k_stream selects and encodes the unit (at most 4096 coordinates, segmented context)
};

// one chunk (multi-segment contexts only).  inblock = 1: the chunk's k_stream block belongs to one unit of at most 4096
// coordinates, which that block also selects and encodes; chunk = NO_CHUNK then pads the unit to a whole block.
// first = the chunk's first coordinate within the row and valid = how many of its 1024 lie inside the unit, so that the
// wave's streaming loads wait for this one record only and not for the segment's as well.
struct WtInfo { uint32_t seg, chunk, first; uint16_t valid, inblock; };
constexpr uint32_t NO_CHUNK = 0xFFFFFFFFu;
struct SelInfo { uint32_t seg, j, pad0, pad1; };                    // one block of a selection kernel
struct CbInfo { uint32_t seg, b, pad0, pad1; };                     // one compaction block

// Every field is written by exactly one kernel of a call and read only by later kernels (the blocks of
// one launch start at different times: a field that a launch both reads and rewrites would show late
// blocks the new value).
struct UnitState {
  uint32_t path;        // static: PATH_FAST, PATH_GENERAL, PATH_SMALL or PATH_FULL
  uint32_t T;           // guess key of this call (k_sample_scan on a cold start; else rolled over from T_next by k_pack;
                        // static for Rand_k and for the general path)
  uint32_t sh;          // the candidates' histogram has bins of 2^sh keys above T (same sources as T)
  uint32_t T_next, sh_next;   // guess and bin width for the next call, from this call's candidates (k_lean_mark)
  uint32_t T_used;      // the guess the last call worked with (k_pack; diagnostics)
  uint32_t cand;        // candidates collected (k_lean_hist)
  uint32_t fell_back;   // 1: the guess failed -- too few candidates or no room for them (k_lean_hist)
  uint32_t crowded;     // 1: the threshold's bin holds more than LISTCAP candidates (k_lean_mark)
  uint32_t taubin, above;     // bin of the k-th largest candidate, candidates in the bins above it (k_lean_mark)
  uint32_t prefix1, k_rem1; // radix selection state after the first digit (found by k_select<1> from the first histogram) ...
  uint32_t prefix2, k_rem2; // ... and after the second (k_select<2>); the third is found by k_tile_count
  uint32_t tau, need, n_gt; // threshold key, how many equal to it are kept, how many above (k_tile_count)
  uint32_t nnz;         // transmitted coordinates (zeroed by k_select<0>, counted by k_quantize)
  uint32_t scale_bits;  // fp32 scale that the message carries (k_quantize, k_lean_emit, ...)
  uint32_t scale_code;  // index-free format only: the scale the codes are computed with (k_dense_scales)
};

struct DevCtx {
  const SegInfo* segs; const WtInfo* wts; const SelInfo* sels; const SelInfo* samps; const CbInfo* cbs;
  const SelInfo* fsels;     // one entry per block of the guessing units' kernels (k_lean_*)
  const uint32_t* fast_segs;
  const uint32_t* small_segs;
  const SelInfo* fulls;     // one entry per block of k_full: (segment with k = size, block number)
  const uint32_t* big_segs; // the segments that are not selected by one block (they use histograms)
  const uint32_t* seg_dir;  // [ceil(d / 1024) + 1]: segment of coordinate t * 1024 (the last entry: L - 1)
  const uint32_t* slot_dir; // [ceil(K / 256) + 1]: segment of slot b * 256 of the selected arrays
  const uint32_t* seg_start; const uint32_t* seg_koff;   // [L]: first coordinate / first slot of every segment, packed for the searches
  const uint32_t* seg_whole;  // [L]: 1 where the segment is kept whole (k = size)
  UnitState* units;
  uint2* slots; uint64_t slot_stride;   // per worker: one slot (lpc * 2 elements) per chunk of every fast segment
  uint2* ovf; uint64_t ovf_stride;      // per worker: overflow pools, for chunks with more candidates than a slot holds
  uint32_t* slot_key; uint32_t* ovf_key; // Rand_k only: the rank key (random word) of every slot element / pool entry
  uint2* d0; uint32_t* d0_key; uint64_t d0_stride;   // per worker: dense, coordinate-ordered candidate lists (+ keys, Rand_k)
  const uint32_t* one_segs; // the guessing segments whose units have a single block: k_lean_one takes them (heaviest first)
  uint32_t* wave_cnt;   // [R][NWC]: candidates met by each wave of k_lean_hist
  uint32_t* wave_sel;   // [R][NWC]: of these, how many lie in the bins above the threshold's (k_lean_mark)
  uint4* tlist;         // [R][nfast][LISTCAP]: the candidates in the threshold's bin: (place in the dense list, value bits, key, -)
  uint32_t* host_flag;  // pinned host memory: set when a failed guess had to be resolved by one block reading the whole unit
  uint2* cb_cnt;        // [R][NCB]: (#key > tau, #key == tau) of each compaction block
  uint32_t* hist;       // [U][3][HBINS], one histogram per radix digit; all zero between calls
  uint32_t* ctr;        // [U][CTR_LINES][PAD]; word 0 of each line is a counter; all zero between calls
  uint64_t* norm_acc;   // [U][ACC_SLOTS]; all zero between calls
  uint32_t* sel_idx; uint32_t* sel_val; uint32_t* sel_code;   // [R][K]; code = level | neg << 31
  uint32_t* blk_cnt;    // [Rmax][QB] transmitted entries per block of 256 slots: added to by every kernel that encodes.  Two arrays
  uint32_t* blk_cnt_next; // take turns from call to call: the last kernel of a call (k_pack) sets the next call's to zero.
  uint32_t* blk_pre;    // [R][QB + 1] their exclusive prefix and total (only when QB > MAX_QB_INLINE)
  uint32_t* surv_idx; uint32_t* surv_code;                    // [R][K]: what k_pack reads (not QSGD, which k_pack_sent packs from sel_*)
  uint64_t* dense_part; // index-free format: [R][ACC_SLOTS][blocks of k_dense_norm] digit sums of every block's first unit ...
  uint32_t* dense_tag;  // ... [R][blocks]: which unit that is, or NO_UNIT
  uint32_t* status;
  uint64_t d, seed;
  uint32_t dense;       // 1: every coordinate is kept and the messages have the index-free format
  uint32_t L, K, NWT, NSEL, NCB, NWC, QB, NSELF, nfast, nblock, Rmax, nbig, s, w_idx, w_lev, w_val, sparsifier, quantizer, cap_words;
  uint32_t none;        // entries of one_segs
};

__device__ __forceinline__ uint32_t key_of_value(uint32_t vbits) { return (vbits & 0x7FFFFFFFu) << 1; }

// Bin of a candidate's key in the histogram of a guessing unit: bins of 2^sh keys counted from the guess T
// (every candidate has key >= T); whatever lies beyond the 4095 bins above T shares the last one.
__device__ __forceinline__ uint32_t lean_bin(uint32_t key, uint32_t T, uint32_t sh) {
  const uint32_t x = (key - T) >> sh;
  return x < HBINS - 1 ? x : HBINS - 1;
}

// quantiser families: QSGD and its scaled form (Lemma 2) share everything but the transmitted norm
__host__ __device__ __forceinline__ bool is_qsgd(uint32_t q) { return q == QSL_QSGD || q == QSL_QSGD_SCALED; }
// which exact sum the quantiser's scale needs: squares (l2 norm), magnitudes (l1 norm), none
__host__ __device__ __forceinline__ bool wants_squares(uint32_t q) { return is_qsgd(q) || q == QSL_SIGN_L2; }
// ... as the power p of sum |v|^p: 2 (QSGD, sign scaled by the l2 norm), 1, 3 or 4 (Lemma 3 with m = 1, 3, 4)
__host__ __device__ __forceinline__ uint32_t norm_power(uint32_t q) {
  return q == QSL_SIGN_L3 ? 3u : q == QSL_SIGN_L4 ? 4u : wants_squares(q) ? 2u : 1u;
}
// How many of the ACC_SLOTS digits the quantiser's sum can reach (squares of fp32 values: 2 * 254 + 48 bits, plus 32
// for their number), and the distance between two accumulator rows in LDS: the kernels clear and add up only these.
__host__ __device__ __forceinline__ uint32_t acc_slots(uint32_t q) { return norm_power(q) <= 2u ? 20u : ACC_SLOTS; }
__host__ __device__ __forceinline__ uint32_t acc_stride(uint32_t q) { return acc_slots(q) + 1u; }

__device__ __forceinline__ uint32_t eff_path(const UnitState& us) {
  return us.path == PATH_FAST && us.fell_back ? static_cast<uint32_t>(PATH_FALLBACK) : us.path;
}

// Find, scanning the first NBINS bins of a histogram from the top, the bin in which the running count
// reaches `target` (1-based).  NT threads (the whole block), thread t owns the NBINS/NT bins below
// NBINS - t * NBINS/NT.  Returns the bin; *above = count in the bins above it.  If the histogram
// holds fewer than `target` entries, returns bin 0 with *above = total - hist[0].  If `clear`,
// zeroes the histogram afterwards.  COPIES > 1: the histogram is the sum of COPIES arrays HBINS apart.
template <uint32_t NT, uint32_t NBINS = HBINS, uint32_t COPIES = 1>
__device__ uint32_t find_from_top(uint32_t* hist, uint32_t target, uint32_t* above, uint64_t* scratch,
                                  uint32_t* result, bool clear) {
  constexpr uint32_t PER = NBINS / NT;
  static_assert(PER >= 1 && PER * NT == NBINS, "bins must divide evenly over the threads");
  const uint32_t t = threadIdx.x;
  uint32_t h[PER]; uint32_t sum = 0;
#pragma unroll
  for (uint32_t j = 0; j < PER; ++j) {
    h[j] = 0;
#pragma unroll
    for (uint32_t cp = 0; cp < COPIES; ++cp) h[j] += hist[cp * HBINS + NBINS - 1 - (PER * t + j)];
    sum += h[j];
  }
  uint64_t total;
  const uint64_t before = block_exclusive_scan64(sum, scratch, &total);
  if (t == NT - 1) { result[0] = 0; result[1] = static_cast<uint32_t>(total) - h[PER - 1]; }
  __syncthreads();
  if (before < target && before + sum >= target) {
    uint32_t cum = static_cast<uint32_t>(before);
#pragma unroll
    for (uint32_t j = 0; j < PER; ++j) {
      if (cum + h[j] >= target) { result[0] = NBINS - 1 - (PER * t + j); result[1] = cum; break; }
      cum += h[j];
    }
  }
  if (clear) {
#pragma unroll
    for (uint32_t j = 0; j < PER; ++j)
      if (h[j]) {
#pragma unroll
        for (uint32_t cp = 0; cp < COPIES; ++cp) hist[cp * HBINS + NBINS - 1 - (PER * t + j)] = 0;
      }
  }
  __syncthreads();
  *above = result[1];
  return result[0];
}

// The same scan for two ranks at once (t0 <= t1).  result[0], result[1]: bin and count above it for t0; result[2],
// result[3]: for t1; result[4]: entries in the bin of t0; result[5]: entries in all.  A rank beyond the total gives
// bin 0 with "above" = total - hist[0], as in find_from_top.
template <uint32_t NT, uint32_t COPIES = 1>
__device__ void find2_from_top(uint32_t* hist, uint32_t t0, uint32_t t1, uint64_t* scratch, uint32_t* result, bool clear) {
  constexpr uint32_t PER = HBINS / NT;
  static_assert(PER >= 1 && PER * NT == HBINS, "bins must divide evenly over the threads");
  const uint32_t t = threadIdx.x;
  uint32_t h[PER]; uint32_t sum = 0;
#pragma unroll
  for (uint32_t j = 0; j < PER; ++j) {
    h[j] = 0;
#pragma unroll
    for (uint32_t cp = 0; cp < COPIES; ++cp) h[j] += hist[cp * HBINS + HBINS - 1 - (PER * t + j)];
    sum += h[j];
  }
  uint64_t total;
  const uint64_t before = block_exclusive_scan64(sum, scratch, &total);
  if (t == NT - 1) {
    const uint32_t rest = static_cast<uint32_t>(total) - h[PER - 1];
    result[0] = 0; result[1] = rest; result[2] = 0; result[3] = rest; result[4] = h[PER - 1]; result[5] = static_cast<uint32_t>(total);
  }
  __syncthreads();
#pragma unroll
  for (uint32_t which = 0; which < 2; ++which) {
    const uint32_t target = which ? t1 : t0;
    if (before < target && before + sum >= target) {
      uint32_t cum = static_cast<uint32_t>(before);
#pragma unroll
      for (uint32_t j = 0; j < PER; ++j) {
        if (cum + h[j] >= target) {
          result[2 * which] = HBINS - 1 - (PER * t + j); result[2 * which + 1] = cum;
          if (which == 0) result[4] = h[j];
          break;
        }
        cum += h[j];
      }
    }
  }
  if (clear) {
#pragma unroll
    for (uint32_t j = 0; j < PER; ++j)
      if (h[j]) {
#pragma unroll
        for (uint32_t cp = 0; cp < COPIES; ++cp) hist[cp * HBINS + HBINS - 1 - (PER * t + j)] = 0;
      }
  }
  __syncthreads();
}

__device__ __forceinline__ void flush_hist(const uint32_t* lh, uint32_t* gh) {
  for (uint32_t i = threadIdx.x; i < HBINS; i += blockDim.x) {
    const uint32_t v = lh[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

}  // namespace
