// qsl_oracle.cpp -- CPU oracle for the Qsparse-local-SGD compression step.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, sequential statement
// of what the error-compensated compression operator computes.  It is used by
// the test-suite, by the smoke check and by the benchmark's CPU-baseline leg,
// and by nothing else; the GPU library never links, imports or calls it, and
// it includes no GPU header and shares no code with the HIP kernels.
//
// What it follows (Basu, Data, Karakus, Diggavi, "Qsparse-local-SGD",
// arXiv:1906.02367):
//   * Algorithm 1, the two worker lines of a synchronisation step:
//       g <- Q Comp_k(m + (x_t - xhat_{t+1/2})),   m <- m + (x_t - xhat) - g,
//     and the master line x_{t+1} = x_t - (1/R) sum_r g^(r).
//   * Section 2.2: Top_k keeps the k largest-magnitude components, Rand_k keeps
//     a uniformly random k-subset.
//   * Definition 1 with example 1 (QSGD, the s-level stochastic quantiser of
//     Alistarh et al.) and Definition 2 (Sign; zero maps to +1).
//   * Lemma 1 and its proof: the quantiser sees the k kept values as a
//     length-k vector (its norm is the norm of the kept values).
//   * Lemma 3 with m = 1: every kept coordinate becomes +-||Comp_k(x)||_1 / k.
//   * Corollary 1: the operator may be applied block by block.
//
// What the paper leaves open and this file fixes (each is a *reading*, listed
// in the design notes of the repository): ties in Top_k go to the lower index;
// Rand_k is "the k coordinates with the largest per-coordinate Philox words";
// level 0 of QSGD is not transmitted; the wire format of a message; norms are
// the correctly rounded value of the exact sum; every written fp32 operation is
// one IEEE round-to-nearest-even operation with denormals kept.
//
// Parity status: the selection, the sign operator, the error update, the
// aggregation and the exact sums are pinned by tests against definitions,
// closed forms and brute force.  The QSGD codes are pinned statistically
// (unbiasedness, second moment) and by deterministic special cases.  The wire
// format, the Rand_k construction and the Philox counter layout are this
// build's own choices: "parity unpinned" by the paper.
//
// Build: g++ -std=c++17 -O2 -ffp-contract=off -fPIC -shared (no -ffast-math, no -march).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <vector>

namespace {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  A counter-based generator: 128-bit counter, 64-bit key,
// ten rounds of two 32x32->64 multiplies and a key bump.
// ---------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
  const uint64_t MUL_A = 0xD2511F53ull, MUL_B = 0xCD9E8D57ull;
  const uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
  uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
  uint32_t k0 = key_in[0], k1 = key_in[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t pa = MUL_A * c0;
    const uint64_t pb = MUL_B * c2;
    const uint32_t n0 = static_cast<uint32_t>(pb >> 32) ^ c1 ^ k0;
    const uint32_t n1 = static_cast<uint32_t>(pb);
    const uint32_t n2 = static_cast<uint32_t>(pa >> 32) ^ c3 ^ k1;
    const uint32_t n3 = static_cast<uint32_t>(pa);
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += WEYL_A; k1 += WEYL_B;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

enum : uint32_t { STREAM_SELECT = 0, STREAM_QUANT = 1 };

// The 32-bit random word attached to coordinate i of `worker` at `round` in
// one of two independent streams.  One Philox block serves four consecutive
// coordinates: counter = (i / 4, worker, round mod 2^32, (round >> 32) | stream << 30),
// key = (seed mod 2^32, seed >> 32); coordinate i takes output word i mod 4.
uint32_t random_word(uint64_t seed, uint32_t worker, uint64_t round, uint32_t stream, uint64_t i) {
  const uint32_t ctr[4] = {static_cast<uint32_t>(i >> 2), worker, static_cast<uint32_t>(round),
                           static_cast<uint32_t>(round >> 32) | (stream << 30)};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  uint32_t out[4];
  philox4x32_10(ctr, key, out);
  return out[i & 3];
}

// ---------------------------------------------------------------------------
// Exact sums.  A wide fixed-point integer (1408 bits: enough for 2^32 fourth powers of
// fp32 values) holds sum_i M_i * 2^{p_i} exactly; it is then rounded once, to nearest-even,
// to a double.
// ---------------------------------------------------------------------------
struct WideInt {
  static const int LIMBS = 22;
  uint64_t limb[LIMBS];
  WideInt() { std::memset(limb, 0, sizeof limb); }
  // add mant * 2^shift  (mant < 2^48, so the shifted value spans at most two limbs)
  void add_shifted(uint64_t mant, unsigned shift) {
    const unsigned w = shift / 64, b = shift % 64;
    uint64_t lo = mant << b;
    uint64_t hi = b ? (mant >> (64 - b)) : 0;
    unsigned j = w;
    uint64_t carry = 0;
    uint64_t t = limb[j] + lo; carry = t < lo; limb[j] = t; ++j;
    t = limb[j] + hi; uint64_t c2 = t < hi; t += carry; c2 |= (t < carry); limb[j] = t; carry = c2; ++j;
    while (carry && j < static_cast<unsigned>(LIMBS)) { limb[j] += 1; carry = (limb[j] == 0); ++j; }
  }
  // add (hi * 2^64 + lo) * 2^shift: the value spans at most three limbs
  void add_shifted128(uint64_t lo, uint64_t hi, unsigned shift) {
    const unsigned w = shift / 64, b = shift % 64;
    const uint64_t part[3] = {lo << b, b ? ((lo >> (64 - b)) | (hi << b)) : hi, b ? (hi >> (64 - b)) : 0};
    uint64_t carry = 0;
    unsigned j = w;
    for (int i = 0; i < 3 && j < static_cast<unsigned>(LIMBS); ++i, ++j) {
      const uint64_t t = limb[j] + part[i];
      const uint64_t c1 = t < part[i];
      const uint64_t t2 = t + carry;
      const uint64_t c2 = t2 < carry;
      limb[j] = t2; carry = c1 | c2;
    }
    while (carry && j < static_cast<unsigned>(LIMBS)) { limb[j] += 1; carry = (limb[j] == 0); ++j; }
  }
  int top_bit() const {  // index of the highest set bit, -1 if zero
    for (int j = LIMBS - 1; j >= 0; --j)
      if (limb[j]) return j * 64 + 63 - __builtin_clzll(limb[j]);
    return -1;
  }
  bool bit(int p) const { return p >= 0 && ((limb[p / 64] >> (p % 64)) & 1u); }
  bool any_below(int p) const {  // any set bit at a position < p
    for (int q = 0; q < p && q < LIMBS * 64; ++q) if (bit(q)) return true;
    return false;
  }
  // value * 2^lsb_exp rounded to nearest-even double (no overflow/underflow in our ranges)
  double to_double(int lsb_exp) const {
    const int h = top_bit();
    if (h < 0) return 0.0;
    uint64_t mant = 0;
    const int low = h - 52;  // position of the last kept bit
    for (int q = h; q >= std::max(low, 0); --q) mant = (mant << 1) | (bit(q) ? 1u : 0u);
    if (low <= 0) return std::ldexp(static_cast<double>(mant), lsb_exp);  // exact
    const bool guard = bit(low - 1);
    const bool sticky = any_below(low - 1);
    if (guard && (sticky || (mant & 1u))) mant += 1;  // may become 2^53: still exact as a double
    return std::ldexp(static_cast<double>(mant), lsb_exp + low);
  }
};

inline uint32_t f2u(float x) { uint32_t u; std::memcpy(&u, &x, 4); return u; }
inline float u2f(uint32_t u) { float x; std::memcpy(&x, &u, 4); return x; }

// |x| = M * 2^E with integer M < 2^24 (valid for finite x, denormals included)
inline void split_abs(float x, uint32_t* M, int* E) {
  const uint32_t u = f2u(x) & 0x7FFFFFFFu;
  const uint32_t e = u >> 23, frac = u & 0x7FFFFFu;
  if (e == 0) { *M = frac; *E = -149; } else { *M = frac | 0x800000u; *E = static_cast<int>(e) - 150; }
}

// RN64( sum_i x_i^2 ) with the sum taken exactly
double exact_sum_of_squares(const float* x, uint64_t n) {
  WideInt acc;
  for (uint64_t i = 0; i < n; ++i) {
    uint32_t M; int E; split_abs(x[i], &M, &E);
    if (M) acc.add_shifted(static_cast<uint64_t>(M) * M, static_cast<unsigned>(2 * E + 298));
  }
  return acc.to_double(-298);
}

// RN64( sum_i |x_i| ) with the sum taken exactly
double exact_sum_of_abs(const float* x, uint64_t n) {
  WideInt acc;
  for (uint64_t i = 0; i < n; ++i) {
    uint32_t M; int E; split_abs(x[i], &M, &E);
    if (M) acc.add_shifted(M, static_cast<unsigned>(E + 149));
  }
  return acc.to_double(-149);
}

// RN64( sum_i |x_i|^p ), p = 3 or 4, with the sum taken exactly (|x|^p = M^p * 2^{p E}, M^p < 2^96)
double exact_sum_of_power(const float* x, uint64_t n, unsigned p) {
  WideInt acc;
  for (uint64_t i = 0; i < n; ++i) {
    uint32_t M; int E; split_abs(x[i], &M, &E);
    if (!M) continue;
    unsigned __int128 P = M;
    for (unsigned j = 1; j < p; ++j) P *= M;
    acc.add_shifted128(static_cast<uint64_t>(P), static_cast<uint64_t>(P >> 64), p * static_cast<unsigned>(E + 149));
  }
  return acc.to_double(-149 * static_cast<int>(p));
}

// Cube root of a positive normal double by a fixed sequence of IEEE operations, so that every implementation that
// performs them one by one gets the same bits: start from 2^floor(E/3) times 1, 2^(1/3) or 2^(2/3) (E the binary
// exponent; at most 26 % below the root), then eight Newton steps y <- (2 y + x / y^2) / 3, each of which squares
// the relative error.  Lemma 3 fixes the norm, not how its root is rounded: this is the reading taken.
double cube_root_fixed(double x) {
  if (!(x > 0.0)) return 0.0;
  uint64_t b; std::memcpy(&b, &x, 8);
  const int E = static_cast<int>(b >> 52) - 1023;
  int q = E / 3, r = E % 3;
  if (r < 0) { r += 3; q -= 1; }
  const uint64_t yb = static_cast<uint64_t>(q + 1023) << 52;
  double y; std::memcpy(&y, &yb, 8);
  y = y * (r == 0 ? 1.0 : r == 1 ? 1.2599210498948732 : 1.5874010519681994);
  for (int it = 0; it < 8; ++it) {
    const double t = y * y;
    const double u = x / t;
    const double w = 2.0 * y;
    y = (w + u) / 3.0;
  }
  return y;
}

// ---------------------------------------------------------------------------
// Wire format helpers
// ---------------------------------------------------------------------------
inline uint32_t bit_width(uint64_t x) {  // bits needed to write x (0 -> 0)
  uint32_t w = 0; while (x) { ++w; x >>= 1; } return w;
}
inline uint32_t index_width(uint64_t d) { return std::max<uint32_t>(1u, bit_width(d - 1)); }
inline uint32_t level_width(uint32_t s) { return bit_width(static_cast<uint64_t>(s) - 1); }

struct BitWriter {
  uint8_t* buf; uint64_t cap_bits; uint64_t pos; bool overflow;
  BitWriter(uint8_t* b, uint64_t cap_bytes) : buf(b), cap_bits(cap_bytes * 8), pos(0), overflow(false) {}
  void put(uint64_t value, uint32_t width) {  // least significant bit first
    for (uint32_t b = 0; b < width; ++b, ++pos) {
      if (pos >= cap_bits) { overflow = true; continue; }
      if ((value >> b) & 1u) buf[pos >> 3] |= static_cast<uint8_t>(1u << (pos & 7));
    }
  }
  void align32() { pos = (pos + 31) / 32 * 32; }
};

struct BitReader {
  const uint8_t* buf; uint64_t pos;
  explicit BitReader(const uint8_t* b) : buf(b), pos(0) {}
  uint64_t get(uint32_t width) {
    uint64_t v = 0;
    for (uint32_t b = 0; b < width; ++b, ++pos)
      v |= static_cast<uint64_t>((buf[pos >> 3] >> (pos & 7)) & 1u) << b;
    return v;
  }
  void align32() { pos = (pos + 31) / 32 * 32; }
};

enum : uint32_t { SPARS_TOPK = 0, SPARS_RANDK = 1 };
// QSGD (Definition 1, example 1); Sign scaled by ||v_S||_1 / k or ||v_S||_2 / k (Lemma 3 with m = 1, 2);
// no quantisation at all (the TopK-SGD comparison scheme of Section 5); QSGD divided by 1 + beta_{k,s} (Lemma 2).
enum : uint32_t { QUANT_QSGD = 0, QUANT_SIGN_L1 = 1, QUANT_SIGN_L2 = 2, QUANT_FP32 = 3, QUANT_QSGD_SCALED = 4,
                  QUANT_SIGN_L3 = 5, QUANT_SIGN_L4 = 6 };
inline bool is_qsgd(uint32_t q) { return q == QUANT_QSGD || q == QUANT_QSGD_SCALED; }
// Added to the quantiser number by the callers of this file: the message has the index-free format of an operator
// that keeps every coordinate (k = size in every segment: the error-feedback schemes without sparsification that
// Section 5 compares with).  Every coordinate has a code, in coordinate order, so no index is written; a QSGD code
// is the level 0..s itself, in the bits needed to write s, then the sign bit.
const uint32_t QUANT_DENSE_FORMAT = 0x100;

struct Layout {
  uint64_t d; uint32_t L; const uint64_t* off; const uint32_t* k; uint32_t s; uint32_t quantizer; bool dense;
  Layout(uint64_t d_, uint32_t L_, const uint64_t* off_, const uint32_t* k_, uint32_t s_, uint32_t quantizer_arg)
      : d(d_), L(L_), off(off_), k(k_), s(s_), quantizer(quantizer_arg & 0xFFu), dense((quantizer_arg & QUANT_DENSE_FORMAT) != 0) {}
  uint64_t K() const { uint64_t t = 0; for (uint32_t l = 0; l < L; ++l) t += k[l]; return t; }
  bool has_counts() const { return is_qsgd(quantizer) && L > 1 && !dense; }
  uint32_t w_idx() const { return dense ? 0 : index_width(d); }
  uint32_t w_val() const {
    if (is_qsgd(quantizer)) return (dense ? bit_width(s) : level_width(s)) + 1;
    return quantizer == QUANT_FP32 ? 32 : 1;
  }
  uint64_t header_bits() const { return 32 + 32ull * L + (has_counts() ? 32ull * L : 0); }
  uint64_t capacity_bytes() const {
    const uint64_t Kt = K();
    uint64_t bits = header_bits();
    bits += (Kt * w_idx() + 31) / 32 * 32;
    bits += (Kt * w_val() + 31) / 32 * 32;
    return (bits + 63) / 64 * 8;
  }
  bool valid() const {
    if (d == 0 || d >= (1ull << 32) || L == 0 || off[0] != 0 || off[L] != d) return false;
    for (uint32_t l = 0; l < L; ++l) {
      if (off[l + 1] <= off[l]) return false;
      if (k[l] == 0 || k[l] > off[l + 1] - off[l]) return false;
    }
    if (is_qsgd(quantizer) && (s == 0 || s > 32768)) return false;
    if (dense) for (uint32_t l = 0; l < L; ++l) if (k[l] != off[l + 1] - off[l]) return false;
    return quantizer <= QUANT_SIGN_L4;
  }
  uint32_t segment_of(uint64_t i) const {
    uint32_t l = 0; while (off[l + 1] <= i) ++l; return l;
  }
};

// dequantised magnitude of QSGD level `lev` under norm N: fl32( fl32(N * lev) / s )
inline float qsgd_magnitude(float N, uint32_t lev, uint32_t s) {
  const float prod = N * static_cast<float>(lev);
  return prod / static_cast<float>(s);
}

}  // namespace

extern "C" {

// -- small exported pieces, so that tests can pin them one by one ------------

void qslo_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) { philox4x32_10(ctr, key, out); }

uint32_t qslo_random_word(uint64_t seed, uint32_t worker, uint64_t round, uint32_t stream, uint64_t i) {
  return random_word(seed, worker, round, stream, i);
}

double qslo_exact_sum_of_squares(const float* x, uint64_t n) { return exact_sum_of_squares(x, n); }
double qslo_exact_sum_of_abs(const float* x, uint64_t n) { return exact_sum_of_abs(x, n); }

uint64_t qslo_msg_capacity_bytes(uint64_t d, uint32_t L, const uint64_t* off, const uint32_t* k, uint32_t s,
                                 uint32_t quantizer) {
  Layout lay(d, L, off, k, s, quantizer);
  return lay.valid() ? lay.capacity_bytes() : 0;
}

// ---------------------------------------------------------------------------
// One worker, one synchronisation round (Algorithm 1, the two worker lines).
//
//   m, delta : d floats each (error memory; accumulated local update)
//   m_out    : d floats or NULL; receives m + delta - g; may alias m
//   msg      : msg_capacity bytes, receives the packed message (zero padded)
//   msg_bits : payload bit count (padding excluded)
//   sel_idx  : K = sum_l k_l selected global indices, ascending inside each segment (may be NULL)
//   sel_level: K entries; QSGD level in {0..s} (0 = not transmitted); 1 for every Sign entry (may be NULL)
//   sel_neg  : K entries, 1 where the kept value is < 0 (may be NULL)
//   scales   : L floats, the per-segment norm N (QSGD) or magnitude c (Sign) (may be NULL)
//   g_val    : K floats, the dequantised value sent for each selected coordinate,
//              0 where nothing is sent (may be NULL)
// Returns 0, or 1 invalid argument, 2 message buffer too small, 3 non-finite input.
// ---------------------------------------------------------------------------
int qslo_compress(const float* m, const float* delta, float* m_out, uint64_t d, uint32_t L, const uint64_t* off,
                  const uint32_t* k, uint32_t s, uint32_t sparsifier, uint32_t quantizer, uint64_t seed,
                  uint32_t worker, uint64_t round, uint8_t* msg, uint64_t msg_capacity, uint64_t* msg_bits,
                  uint32_t* sel_idx, uint16_t* sel_level, uint8_t* sel_neg, float* scales, float* g_val) {
  Layout lay(d, L, off, k, s, quantizer);
  quantizer = lay.quantizer;                        // without the format flag
  if (!m || !delta || !msg || !lay.valid() || sparsifier > 1 || (round >> 62)) return 1;
  if (msg_capacity < lay.capacity_bytes()) return 2;
  const uint64_t K = lay.K();

  // Step 1 (Algorithm 1, worker line 1): the error-compensated update v = m + delta.
  std::vector<float> v(d);
  for (uint64_t i = 0; i < d; ++i) {
    v[i] = m[i] + delta[i];
    if ((f2u(v[i]) & 0x7FFFFFFFu) >= 0x7F800000u) return 3;
  }

  std::vector<uint32_t> S(K);        // selected indices
  std::vector<uint16_t> lev(K, 0);   // QSGD level, or 1 for every Sign entry
  std::vector<uint8_t> neg(K, 0);    // 1{v_i < 0}
  std::vector<float> g(K, 0.0f);     // value sent (0: nothing sent)
  std::vector<float> scale(L, 0.0f);
  std::vector<uint32_t> nnz(L, 0);

  uint64_t base = 0;
  for (uint32_t l = 0; l < L; ++l) {
    const uint64_t lo = off[l], n = off[l + 1] - off[l];
    const uint32_t kl = k[l];

    // Step 2 (Section 2.2): choose the index set.  Each coordinate gets a 32-bit
    // rank key -- the magnitude bits of v_i for Top_k, its SELECT-stream random
    // word for Rand_k -- and the k_l coordinates that come first under
    // (key descending, index ascending) are kept.
    std::vector<uint64_t> order(n);
    for (uint64_t j = 0; j < n; ++j) {
      const uint64_t i = lo + j;
      const uint32_t key = sparsifier == SPARS_TOPK ? (f2u(v[i]) & 0x7FFFFFFFu)
                                                    : random_word(seed, worker, round, STREAM_SELECT, i);
      order[j] = (static_cast<uint64_t>(key) << 32) | (0xFFFFFFFFu - static_cast<uint32_t>(i));
    }
    if (n <= 256) std::sort(order.begin(), order.end(), std::greater<uint64_t>());
    else std::nth_element(order.begin(), order.begin() + (kl - 1), order.end(), std::greater<uint64_t>());
    uint32_t* Sl = S.data() + base;
    for (uint32_t j = 0; j < kl; ++j) Sl[j] = 0xFFFFFFFFu - static_cast<uint32_t>(order[j]);
    std::sort(Sl, Sl + kl);

    // the kept values as a length-k_l vector (proof of Lemma 1)
    std::vector<float> vs(kl);
    for (uint32_t j = 0; j < kl; ++j) vs[j] = v[Sl[j]];

    if (is_qsgd(quantizer)) {
      // Step 3: N = || v_S ||_2, the exact sum rounded to double, square root, rounded to float.
      const float N = static_cast<float>(std::sqrt(exact_sum_of_squares(vs.data(), kl)));
      // Lemma 2: the scaled operator sends Q_s(v_S) / (1 + beta_{k,s}), beta_{k,s} = min(k / s^2, sqrt(k) / s):
      // the level codes are those of the unscaled operator, the transmitted norm is N / (1 + beta).
      float N_sent = N;
      if (quantizer == QUANT_QSGD_SCALED) {
        const double beta = std::min(static_cast<double>(kl) / (static_cast<double>(s) * s),
                                     std::sqrt(static_cast<double>(kl)) / s);
        N_sent = N / static_cast<float>(1.0 + beta);
      }
      scale[l] = N_sent;
      // Step 4 (Definition 1, example 1): stochastic rounding of s|v_i|/N to one of
      // the two neighbouring integers, up with probability equal to the fraction.
      for (uint32_t j = 0; j < kl; ++j) {
        const float x = vs[j];
        uint32_t level = 0;
        if (N > 0.0f) {
          const float a = std::fabs(x) / N;
          float t = a * static_cast<float>(s);
          if (t > static_cast<float>(s)) t = static_cast<float>(s);
          const float fl = std::floor(t);
          const float frac = t - fl;
          const uint32_t w = random_word(seed, worker, round, STREAM_QUANT, Sl[j]);
          const float u = static_cast<float>(w >> 8) * 0x1p-24f;
          level = static_cast<uint32_t>(fl) + (u < frac ? 1u : 0u);
        }
        lev[base + j] = static_cast<uint16_t>(level);
        neg[base + j] = x < 0.0f;
        if (level) {
          const float mag = qsgd_magnitude(N_sent, level, s);
          g[base + j] = neg[base + j] ? -mag : mag;
          ++nnz[l];
        }
      }
    } else if (quantizer == QUANT_FP32) {
      // no quantiser: g = Top_k(v) (or Rand_k(v)) itself
      scale[l] = 0.0f;
      for (uint32_t j = 0; j < kl; ++j) { neg[base + j] = vs[j] < 0.0f; lev[base + j] = 1; g[base + j] = vs[j]; }
      nnz[l] = kl;
    } else {
      // Step 3 (Lemma 3): c = || v_S ||_m / k, m = 1 .. 4: the exact sum of the m-th powers rounded to double,
      // its m-th root in double, the division by k in double, one rounding to float.
      double norm;
      if (quantizer == QUANT_SIGN_L1) norm = exact_sum_of_abs(vs.data(), kl);
      else if (quantizer == QUANT_SIGN_L2) norm = std::sqrt(exact_sum_of_squares(vs.data(), kl));
      else if (quantizer == QUANT_SIGN_L3) norm = cube_root_fixed(exact_sum_of_power(vs.data(), kl, 3));
      else norm = std::sqrt(std::sqrt(exact_sum_of_power(vs.data(), kl, 4)));
      const float c = static_cast<float>(norm / static_cast<double>(kl));
      scale[l] = c;
      // Step 4 (Definition 2): +c where v_i >= 0 (zero included), -c where v_i < 0.
      for (uint32_t j = 0; j < kl; ++j) {
        neg[base + j] = vs[j] < 0.0f;
        lev[base + j] = 1;
        g[base + j] = neg[base + j] ? -c : c;
      }
      nnz[l] = kl;
    }
    base += kl;
  }

  // Step 5: the message.  [u32 nnz][f32 scale x L][u32 nnz_l x L, QSGD with L > 1 only]
  // [indices of transmitted coordinates, w_idx bits each][codes, w_val bits each];
  // each of the two packed sections starts on a 32-bit boundary.
  std::memset(msg, 0, msg_capacity);
  BitWriter bw(msg, msg_capacity);
  uint64_t total = 0;
  for (uint32_t l = 0; l < L; ++l) total += nnz[l];
  bw.put(lay.dense ? K : total, 32);
  for (uint32_t l = 0; l < L; ++l) bw.put(f2u(scale[l]), 32);
  if (lay.has_counts()) for (uint32_t l = 0; l < L; ++l) bw.put(nnz[l], 32);
  if (lay.dense) {
    // every coordinate, in order: no indices; a QSGD level is written as it is (0 included)
    total = K;
    const uint32_t wl = bit_width(s);
    for (uint64_t j = 0; j < K; ++j) {
      if (is_qsgd(quantizer)) { bw.put(lev[j], wl); bw.put(neg[j], 1); }
      else if (quantizer == QUANT_FP32) bw.put(f2u(g[j]), 32);
      else bw.put(neg[j], 1);
    }
  } else {
    const uint32_t wi = lay.w_idx(), wl = is_qsgd(quantizer) ? level_width(s) : 0;
    for (uint64_t j = 0; j < K; ++j) if (lev[j]) bw.put(S[j], wi);
    bw.align32();
    for (uint64_t j = 0; j < K; ++j) {
      if (!lev[j]) continue;
      if (is_qsgd(quantizer)) { bw.put(lev[j] - 1u, wl); bw.put(neg[j], 1); }
      else if (quantizer == QUANT_FP32) bw.put(f2u(g[j]), 32);
      else bw.put(neg[j], 1);
    }
  }
  if (bw.overflow) return 2;
  if (msg_bits) *msg_bits = lay.header_bits() + total * (lay.w_idx() + lay.w_val());

  // Step 6 (Algorithm 1, worker line 2): m <- v - g.  Off the transmitted set this is v itself.
  if (m_out) {
    for (uint64_t i = 0; i < d; ++i) m_out[i] = v[i];
    for (uint64_t j = 0; j < K; ++j) if (lev[j]) m_out[S[j]] = v[S[j]] - g[j];
  }

  if (sel_idx) std::copy(S.begin(), S.end(), sel_idx);
  if (sel_level) std::copy(lev.begin(), lev.end(), sel_level);
  if (sel_neg) std::copy(neg.begin(), neg.end(), sel_neg);
  if (scales) std::copy(scale.begin(), scale.end(), scales);
  if (g_val) std::copy(g.begin(), g.end(), g_val);
  return 0;
}

// Payload bit count read back from a message.
uint64_t qslo_bits_sent(const uint8_t* msg, uint64_t d, uint32_t L, const uint64_t* off, const uint32_t* k,
                        uint32_t s, uint32_t quantizer) {
  Layout lay(d, L, off, k, s, quantizer);
  BitReader br(msg);
  const uint64_t total = br.get(32);
  return lay.header_bits() + total * (lay.w_idx() + lay.w_val());
}

// Unpack a message into (index, value) pairs; returns the number of pairs, or -1 if
// `max_out` is too small or the message is inconsistent.
int64_t qslo_decode(const uint8_t* msg, uint64_t d, uint32_t L, const uint64_t* off, const uint32_t* k, uint32_t s,
                    uint32_t quantizer, uint32_t* idx_out, float* val_out, uint64_t max_out) {
  Layout lay(d, L, off, k, s, quantizer);
  quantizer = lay.quantizer;
  if (!lay.valid()) return -1;
  BitReader br(msg);
  const uint64_t total = br.get(32);
  if (total > max_out || total > lay.K()) return -1;
  if (lay.dense && total != 0 && total != d) return -1;
  std::vector<float> scale(L);
  for (uint32_t l = 0; l < L; ++l) scale[l] = u2f(static_cast<uint32_t>(br.get(32)));
  if (lay.has_counts()) for (uint32_t l = 0; l < L; ++l) br.get(32);
  const uint32_t wi = lay.w_idx(), wl = is_qsgd(quantizer) ? (lay.dense ? bit_width(s) : level_width(s)) : 0;
  for (uint64_t j = 0; j < total; ++j) idx_out[j] = lay.dense ? static_cast<uint32_t>(j) : static_cast<uint32_t>(br.get(wi));
  br.align32();
  for (uint64_t j = 0; j < total; ++j) {
    if (idx_out[j] >= d) return -1;
    const float sc = scale[lay.segment_of(idx_out[j])];
    if (is_qsgd(quantizer)) {
      const uint32_t level = static_cast<uint32_t>(br.get(wl)) + (lay.dense ? 0u : 1u);
      const bool negative = br.get(1);
      const float mag = qsgd_magnitude(sc, level, s);
      val_out[j] = level == 0 ? 0.0f : negative ? -mag : mag;
    } else if (quantizer == QUANT_FP32) {
      val_out[j] = u2f(static_cast<uint32_t>(br.get(32)));
    } else {
      val_out[j] = br.get(1) ? -sc : sc;
    }
  }
  return static_cast<int64_t>(total);
}

// Stand-alone error update (Algorithm 1, worker line 2) from a message: m <- (m + delta) - decode(msg).
int qslo_error_update(float* m, const float* delta, const uint8_t* msg, uint64_t d, uint32_t L, const uint64_t* off,
                      const uint32_t* k, uint32_t s, uint32_t quantizer) {
  Layout lay(d, L, off, k, s, quantizer);
  if (!lay.valid()) return 1;
  const uint64_t K = lay.K();
  std::vector<uint32_t> idx(K); std::vector<float> val(K);
  const int64_t n = qslo_decode(msg, d, L, off, k, s, quantizer, idx.data(), val.data(), K);
  if (n < 0) return 1;
  for (uint64_t i = 0; i < d; ++i) m[i] = m[i] + delta[i];
  for (int64_t j = 0; j < n; ++j) m[idx[j]] = m[idx[j]] - val[j];
  return 0;
}

// Master line of Algorithm 1: out_j = (accumulate ? out_j : 0) + scale * sum_r decode(msg_r)_j,
// the sum over r in ascending order of the list, accumulated in double.
int qslo_aggregate(const uint8_t* msgs, uint64_t msg_stride, const uint32_t* list, uint32_t R, float scale,
                   int accumulate, float* out, uint64_t d, uint32_t L, const uint64_t* off, const uint32_t* k,
                   uint32_t s, uint32_t quantizer) {
  Layout lay(d, L, off, k, s, quantizer);
  if (!lay.valid()) return 1;
  const uint64_t K = lay.K();
  std::vector<double> acc(d, 0.0);
  std::vector<uint32_t> idx(K); std::vector<float> val(K);
  for (uint32_t q = 0; q < R; ++q) {
    const uint32_t r = list ? list[q] : q;
    const int64_t n = qslo_decode(msgs + msg_stride * r, d, L, off, k, s, quantizer, idx.data(), val.data(), K);
    if (n < 0) return 1;
    for (int64_t j = 0; j < n; ++j) acc[idx[j]] += static_cast<double>(val[j]);
  }
  for (uint64_t i = 0; i < d; ++i) {
    const double prev = accumulate ? static_cast<double>(out[i]) : 0.0;
    out[i] = static_cast<float>(prev + static_cast<double>(scale) * acc[i]);
  }
  return 0;
}

}  // extern "C"
