// fbsr_oracle.cpp -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, serial CPU statement of few-bit stochastic rounding (FBSR),
// written from "On Stochastic Rounding with Few Random Bits" (arXiv 2504.20634)
// in the paper's real-number form: every step is exact arithmetic on doubles
// (frexp/ldexp/floor of values with at most 24 significant bits), never a
// manipulation of the fp32 bit pattern.  It exists so that tests, the smoke
// check and the benchmark's CPU-baseline leg can compare the GPU library
// against something that can be checked against the paper by eye.  The GPU
// library never links, loads or calls it, and the two share no source.
//
// Paper passages followed:
//   format model F(s,e,t;P,B), subnormals at e=0 ............ Sec. II, Eq. (1)
//   exponent  e~ = max(floor(log2 x~), 1-B) .................. Sec. II-A, Eq. (2)
//   scaled significand  s~ = x~ * 2^-e~ * 2^(P-1) ............ Sec. II-A, Eq. (3)
//   sigma = floor(s~) + 1[R(s~ - floor(s~))] ................. Sec. II-A, Eq. (5)
//   R_TNE (ties to nearest even), R_TNO (odd), R_TA (away) ... Sec. II-A, Eq. (4)
//   R_SRFF(d,n) = d + n 2^-N >= 1 ............................ Sec. II-B
//   R_SRF (d,n) = d + (n+1/2) 2^-N >= 1 ...................... Sec. II-B
//   R_SRC (d,n) = R_SRFF(Round(d 2^N) 2^-N, n) ............... Sec. III-F, Eq. (7)
//   out-of-range values round deterministically (IEEE RN) .... Sec. II
//   weight update "w <- RoundTo(w + u), SR applied here" ..... Sec. III, Alg. 1
//   per-input mean of rounded samples, bias in target ulps ... Fig. 1, Fig. 2, Sec. III
//
// Readings taken where the paper is silent (each is also listed in the design notes):
//   * negative inputs: |x| is rounded and the sign re-applied (the paper rounds x~ > 0);
//   * NaN -> the target's canonical quiet NaN with x's sign; +-0 -> +-0;
//   * |x| > M: bf16 / E5M2 round to nearest on the unbounded-exponent grid
//     (below M + ulp(M)/2 -> M, otherwise -> inf; the tie goes to inf because
//     M's significand is odd); E4M3 has no infinity and saturates to +-M;
//   * SRC's inner Round is round-to-nearest, ties to even (ties to odd, which Sec. III-F also
//     allows, is a separate variant of the generic-format entry points);
//   * generic formats (any (K, P, B; M) of Sec. II with K <= 8): special encodings, the absence of
//     -0 and the overflow policy are part of the caller's descriptor (see Format8);
//   * the N random bits of element i are a slice of a Philox4x32-10 block
//     (Salmon et al., SC'11) -- the paper leaves the generator open; the
//     slicing convention is this build's and is restated in random_bits().
//
// Parity pins (tests/test_oracle_*.py): bracketing neighbours, identity on
// representable inputs, N >= D gives exact SR, exhaustive expectations over all
// 2^N draws, the closed-form biases of Sec. III / App. A, Fig. 1's -0.124 and
// Fig. 2's printed biases, RNE against a library cast, Philox known answers.
// Unpinned by anything outside this build: which slice of which Philox block an
// element receives (a convention; the paper fixes no generator).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

namespace {

// ---------------------------------------------------------------- formats ---
// (K, P, B; M) of Sec. II.  has_inf: the format encodes infinities.
struct Format {
  int K;         // width in bits
  int P;         // precision (one more than the stored trailing bits)
  int B;         // exponent bias
  double M;      // largest finite value
  bool has_inf;  // e = all-ones, t = 0 is +-inf
  uint32_t nan_code;  // canonical quiet NaN, sign bit clear
  uint32_t inf_code;  // +inf (unused when !has_inf)
  // A format whose specials do not follow the two patterns above (a NaN that is a sign bit alone,
  // no negative zero, finite values in the top exponent) is rounded and decoded through its
  // generic descriptor (see Format8); nan_code then holds the full NaN code.
  bool by_descriptor = false;
  int32_t desc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
};

enum { FMT_BF16 = 0, FMT_E4M3 = 1, FMT_E5M2 = 2, FMT_BINARY8P4 = 3,
       FMT_FP16 = 16 };   // FP16: IEEE binary16, used as a SOURCE format only (never a caller's target id)
enum { SRC_BF16 = 0, SRC_FP16 = 1 };
enum { VAR_RNE = 0, VAR_SRFF = 1, VAR_SRF = 2, VAR_SRC = 3,
       VAR_SRC_ODD = 4, VAR_TNO = 5, VAR_TA = 6 };   // 4..6: generic-format entry points only

bool get_format(int fmt, Format* f) {
  switch (fmt) {
    case FMT_BF16:  // (2 - 2^-7) * 2^127
      *f = Format{16, 8, 127, std::ldexp(2.0 - std::ldexp(1.0, -7), 127), true, 0x7FC0u, 0x7F80u};
      return true;
    case FMT_E4M3:  // OCP E4M3: finite-only, S.1111.111 is NaN, max 1.75 * 2^8
      *f = Format{8, 4, 7, 448.0, false, 0x7Fu, 0u};
      return true;
    case FMT_E5M2:  // OCP E5M2: IEEE-like, max 1.75 * 2^15
      *f = Format{8, 3, 15, 57344.0, true, 0x7Eu, 0x7Cu};
      return true;
    case FMT_BINARY8P4: {  // IEEE WG P3109 binary8p4, the format Sec. IV trains in: bias 8, max 1.75 * 2^7,
                           // 0x7F / 0xFF infinities, 0x80 the only NaN, no negative zero
      *f = Format{8, 4, 8, 224.0, true, 0x80u, 0x7Fu};
      f->by_descriptor = true;
      const int32_t d[8] = {8, 4, 8, 0x7E, 0x7F, 0x80, 0, 0};
      for (int k = 0; k < 8; ++k) f->desc[k] = d[k];
      return true;
    }
    case FMT_FP16:  // IEEE binary16: (2 - 2^-10) * 2^15
      *f = Format{16, 11, 15, 65504.0, true, 0x7E00u, 0x7C00u};
      return true;
  }
  return false;
}

double decode_by_descriptor(uint32_t code, const Format& f);
uint32_t round_by_descriptor(double xv, const Format& f, int variant, int N, uint64_t n);

// Eq. (1): the real value of (s,e,t); specials per format.
double decode(uint32_t code, const Format& f) {
  if (f.by_descriptor) return decode_by_descriptor(code, f);
  const int tbits = f.P - 1;
  const uint32_t s = (code >> (f.K - 1)) & 1u;
  const uint32_t e = (code >> tbits) & ((1u << (f.K - 1 - tbits)) - 1u);
  const uint32_t t = code & ((1u << tbits) - 1u);
  const uint32_t emax = (1u << (f.K - 1 - tbits)) - 1u;
  const double sign = s ? -1.0 : 1.0;
  if (f.has_inf && e == emax) {
    if (t == 0) return sign * std::numeric_limits<double>::infinity();
    return std::numeric_limits<double>::quiet_NaN();
  }
  if (!f.has_inf && (code & ((1u << (f.K - 1)) - 1u)) == f.nan_code)
    return std::numeric_limits<double>::quiet_NaN();
  if (e == 0) return sign * std::ldexp((double)t, 1 - f.P) * std::ldexp(1.0, 1 - f.B);
  return sign * (1.0 + std::ldexp((double)t, 1 - f.P)) * std::ldexp(1.0, (int)e - f.B);
}

// Encode the non-negative finite value sigma * 2^(et - P + 1), sigma an integer in
// [0, 2^P], et >= 1 - B, value <= M  (Sec. II-A: the trailing bits of sigma are
// stored, the exponent is incremented when sigma = 2^P).
uint32_t encode_magnitude(int64_t sigma, int et, const Format& f) {
  if (sigma == ((int64_t)1 << f.P)) {
    sigma = (int64_t)1 << (f.P - 1);
    et += 1;
  }
  uint32_t e, t;
  if (sigma < ((int64_t)1 << (f.P - 1))) {  // subnormal (only when et == 1 - B) or zero
    e = 0;
    t = (uint32_t)sigma;
  } else {
    e = (uint32_t)(et + f.B);
    t = (uint32_t)(sigma - ((int64_t)1 << (f.P - 1)));
  }
  return (e << (f.P - 1)) | t;
}

// Eq. (2): e~ = max(floor(log2 a), 1 - B) for finite a > 0; a = 0 takes the floor 1 - B.
int rounding_exponent(double a, const Format& f) {
  if (a == 0.0) return 1 - f.B;
  const int lg = std::ilogb(a);  // exact floor(log2 a) for finite positive a
  return lg > 1 - f.B ? lg : 1 - f.B;
}

// ------------------------------------------------------------- predicates ---
// All comparisons are in a form whose two sides are exactly representable:
// delta has at most 24 + (tiny-exponent shift) significant bits but only ever
// appears alone on one side; the other side is a dyadic with <= 26 bits.
bool round_up(int variant, double fl, double delta, int N, uint64_t n) {
  switch (variant) {
    case VAR_RNE:  // R_TNE: delta > 1/2, or a tie and floor+1 is even
      return delta > 0.5 || (delta == 0.5 && std::fmod(fl, 2.0) == 1.0);
    case VAR_SRFF:  // delta + n 2^-N >= 1
      return delta >= 1.0 - std::ldexp((double)n, -N);
    case VAR_SRF:  // delta + (n + 1/2) 2^-N >= 1
      return delta >= 1.0 - std::ldexp((double)(2 * n + 1), -(N + 1));
    case VAR_SRC: {  // SRFF applied to Round(delta 2^N) 2^-N, Round = RN ties-to-even
      const double h = std::nearbyint(std::ldexp(delta, N));  // default FE_TONEAREST
      return h + (double)n >= std::ldexp(1.0, N);
    }
    case VAR_SRC_ODD: {  // the same with Round = RN ties-to-odd (Sec. III-F: "ties to even or odd")
      const double s = std::ldexp(delta, N);
      const double lo = std::floor(s);
      const double r = s - lo;  // exact
      double h = lo;
      if (r > 0.5 || (r == 0.5 && std::fmod(lo, 2.0) == 0.0)) h = lo + 1.0;
      return h + (double)n >= std::ldexp(1.0, N);
    }
    case VAR_TNO:  // R_TNO: a tie goes to the odd neighbour
      return delta > 0.5 || (delta == 0.5 && std::fmod(fl, 2.0) == 0.0);
    case VAR_TA:  // Eq. (4): R_TA(delta) = delta >= 1/2
      return delta >= 0.5;
  }
  return false;
}

// One element: a value with at most 24 significant bits (an fp32 value, or one scaled exactly by a
// power of two) -> code of the target format, given the integer n < 2^N.
uint32_t round_one(double xv, const Format& f, int variant, int N, uint64_t n) {
  if (f.by_descriptor) return round_by_descriptor(xv, f, variant, N, n);
  const uint32_t sign_code = (std::signbit(xv) ? 1u : 0u) << (f.K - 1);
  if (std::isnan(xv)) return sign_code | f.nan_code;
  const double a = std::fabs(xv);
  if (a == 0.0) return sign_code;
  if (a > f.M) {  // outside the finite range: deterministic
    const int eM = std::ilogb(f.M);
    const uint32_t m_code = encode_magnitude((int64_t)std::ldexp(f.M, -eM + f.P - 1), eM, f);  // M is on the grid
    if (!f.has_inf) return sign_code | m_code;  // saturating format
    const double half_ulp_M = std::ldexp(1.0, eM - f.P + 1) / 2.0;
    return sign_code | (a < f.M + half_ulp_M ? m_code : f.inf_code);
  }
  const int et = rounding_exponent(a, f);                   // Eq. (2)
  const double sig = std::ldexp(a, -et + f.P - 1);          // Eq. (3), exact
  const double fl = std::floor(sig);
  const double delta = sig - fl;                            // exact
  const int64_t sigma = (int64_t)fl + (round_up(variant, fl, delta, N, n) ? 1 : 0);  // Eq. (5)
  return sign_code | encode_magnitude(sigma, et, f);
}


// ------------------------------------------------ generic formats, K <= 8 ---
// Any (K, P, B; M) of Sec. II whose codes fit a byte.  The paper's format model says nothing about
// special encodings, so they are data of the descriptor:
//   max_code    magnitude code (e << (P-1) | t) of M; every magnitude code above it is not finite
//   inf_code    magnitude code of infinity, or -1: the format has none and SATURATES (every
//               |x| > M, infinities included, becomes +-M)
//   nan_code    full code of the canonical NaN, or -1: no NaN (a NaN input then becomes +-M)
//   nan_signed  the sign of a NaN input is OR-ed into nan_code
//   neg_zero    the format has -0; without it a negative input that rounds to zero gives code 0
// With an infinity, |x| > M rounds to nearest on the unbounded-exponent grid, ties to even
// (Sec. II: "as in IEEE-754 round to nearest"): below M + ulp(M)/2 -> M, above -> inf, the tie
// to whichever of the two has the even significand.
struct Format8 {
  Format f;   // K, P, B, M (the other fields of f are unused on this path)
  int max_code, inf_code, nan_code;
  bool nan_signed, neg_zero;
};

// desc: {K, P, B, max_code, inf_code, nan_code, nan_signed, neg_zero}.
// max_width: 8 for the entry points whose codes are bytes, 16 for those with 16-bit codes (the format model of
// Sec. II, Eq. (1) is the same at every width; B may then reach 127).
bool get_format8(const int32_t* d, Format8* g, int max_width = 8) {
  const int K = d[0], P = d[1], B = d[2];
  if (K < 2 || K > max_width || P < 1 || P > K - 1 || B < 0 || B > (max_width > 8 ? 127 : 96)) return false;
  const int mag_top = (1 << (K - 1)) - 1;
  const int max_code = d[3], inf_code = d[4], nan_code = d[5];
  if (max_code < (1 << (P - 1)) || max_code > mag_top) return false;        // M is a normal value
  if (inf_code != -1 && (inf_code <= max_code || inf_code > mag_top)) return false;
  const bool nan_signed = d[6] != 0, neg_zero = d[7] != 0;
  if (nan_code != -1) {
    if (nan_code < 0 || nan_code >= (1 << K)) return false;
    const int mag = nan_code & mag_top, sgn = nan_code >> (K - 1);
    const bool above = mag > max_code && mag != inf_code;                   // an unused magnitude
    const bool minus_zero_slot = mag == 0 && sgn == 1 && !neg_zero && !nan_signed;
    if (!above && !minus_zero_slot) return false;
    if (nan_signed && sgn != 0) return false;
  }
  const int e_max = (max_code >> (P - 1)), t_max = max_code & ((1 << (P - 1)) - 1);
  if (e_max - B > 126) return false;                                        // M + ulp(M) must be a finite fp32
  const double M = (1.0 + std::ldexp((double)t_max, 1 - P)) * std::ldexp(1.0, e_max - B);   // Eq. (1), e > 0
  g->f = Format{K, P, B, M, false, 0u, 0u};
  g->max_code = max_code;
  g->inf_code = inf_code;
  g->nan_code = nan_code;
  g->nan_signed = nan_signed;
  g->neg_zero = neg_zero;
  return true;
}

double decode8(uint32_t code, const Format8& g) {
  const Format& f = g.f;
  const uint32_t sign_bit = 1u << (f.K - 1);
  code &= (sign_bit << 1) - 1u;
  const uint32_t mag = code & (sign_bit - 1u);
  const bool neg = (code & sign_bit) != 0;
  const double qnan = std::numeric_limits<double>::quiet_NaN();
  if (g.nan_code >= 0 && (g.nan_signed ? mag == (uint32_t)g.nan_code : code == (uint32_t)g.nan_code)) return qnan;
  if (g.inf_code >= 0 && mag == (uint32_t)g.inf_code)
    return neg ? -std::numeric_limits<double>::infinity() : std::numeric_limits<double>::infinity();
  if (mag > (uint32_t)g.max_code) return qnan;          // an encoding the descriptor leaves unused
  if (mag == 0 && neg && !g.neg_zero) return qnan;      // likewise
  const uint32_t e = mag >> (f.P - 1), t = mag & ((1u << (f.P - 1)) - 1u);
  const double sign = neg ? -1.0 : 1.0;
  if (e == 0) return sign * std::ldexp((double)t, 1 - f.P) * std::ldexp(1.0, 1 - f.B);      // Eq. (1)
  return sign * (1.0 + std::ldexp((double)t, 1 - f.P)) * std::ldexp(1.0, (int)e - f.B);
}

uint32_t round_one8(double xv, const Format8& g, int variant, int N, uint64_t n) {
  const Format& f = g.f;
  const uint32_t sign_code = (std::signbit(xv) ? 1u : 0u) << (f.K - 1);
  if (std::isnan(xv)) {
    if (g.nan_code < 0) return sign_code | (uint32_t)g.max_code;
    return (uint32_t)g.nan_code | (g.nan_signed ? sign_code : 0u);
  }
  const double a = std::fabs(xv);
  if (a == 0.0) return g.neg_zero ? sign_code : 0u;
  if (a > f.M) {  // outside the finite range: deterministic
    if (g.inf_code < 0) return sign_code | (uint32_t)g.max_code;
    const double ulp_M = std::ldexp(1.0, std::ilogb(f.M) - f.P + 1);
    const double tie = f.M + ulp_M / 2.0;
    bool to_inf = a > tie;
    if (a == tie) to_inf = std::fmod(f.M / ulp_M, 2.0) == 1.0;   // M's significand is odd: inf is the even side
    return sign_code | (uint32_t)(to_inf ? g.inf_code : g.max_code);
  }
  const int et = rounding_exponent(a, f);                   // Eq. (2)
  const double sig = std::ldexp(a, -et + f.P - 1);          // Eq. (3), exact
  const double fl = std::floor(sig);
  const double delta = sig - fl;                            // exact
  const int64_t sigma = (int64_t)fl + (round_up(variant, fl, delta, N, n) ? 1 : 0);  // Eq. (5)
  const uint32_t mag = encode_magnitude(sigma, et, f);
  if (mag == 0 && !g.neg_zero) return 0u;
  return sign_code | mag;
}

double decode_by_descriptor(uint32_t code, const Format& f) {
  Format8 g;
  get_format8(f.desc, &g);
  return decode8(code, g);
}

uint32_t round_by_descriptor(double xv, const Format& f, int variant, int N, uint64_t n) {
  Format8 g;
  get_format8(f.desc, &g);
  return round_one8(xv, g, variant, N, n);
}

bool variant8_ok(int variant, int nbits) {
  if (variant < VAR_RNE || variant > VAR_TA) return false;
  const bool draws = variant == VAR_SRFF || variant == VAR_SRF || variant == VAR_SRC || variant == VAR_SRC_ODD;
  return !draws || (nbits >= 1 && nbits <= 32);
}

bool variant_draws(int variant) {
  return variant == VAR_SRFF || variant == VAR_SRF || variant == VAR_SRC || variant == VAR_SRC_ODD;
}

// ----------------------------------------------------------------- Philox ---
// Philox4x32-10 as published (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of
//   (c0,c1,c2,c3) <- (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1, lo(M0 c0))
// with the key bumped by the Weyl constants between rounds.
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53ull, M1 = 0xCD9E8D57ull;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = M0 * c0;
    const uint64_t p1 = M1 * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Slot width: the smallest power of two >= N (1, 2, 4, 8, 16 or 32).
int slot_width(int N) {
  int W = 1;
  while (W < N) W *= 2;
  return W;
}

// This build's convention for "the N random bits of element i" (global index
// i, stream selected by (seed, step)):  a Philox block is 128 bits, words
// out[0..3] little-endian (out[0] holds bits 0..31); it is cut into 128/W
// slots of W bits; element i uses slot i mod (128/W) of block floor(i / (128/W));
// n is the low N bits of its slot.  Counter = (block lo, block hi, step lo,
// step hi), key = (seed lo, seed hi).
uint64_t random_bits(uint64_t seed, uint64_t step, uint64_t i, int N) {
  const int W = slot_width(N);
  const uint64_t per_block = 128u / (unsigned)W;
  const uint64_t blk = i / per_block;
  const unsigned slot = (unsigned)(i % per_block);
  const uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step, (uint32_t)(step >> 32)};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t r[4];
  philox4x32_10(ctr, key, r);
  const unsigned bit = slot * (unsigned)W;
  const uint64_t word = r[bit / 32];
  const uint64_t mask = (N >= 64) ? ~0ull : ((1ull << N) - 1ull);
  return (word >> (bit % 32)) & mask;
}

// The exact fp32 value of a 16-bit source code (bf16 or IEEE binary16) by Eq. (1); every such
// value is representable in fp32.  The sign of zeros, infinities and NaNs is kept.
float widen16(uint16_t code, int src_fmt) {
  Format f;
  get_format(src_fmt == SRC_BF16 ? FMT_BF16 : FMT_FP16, &f);
  const double v = decode(code, f);
  const bool neg = (code >> 15) & 1u;
  if (std::isnan(v)) return std::copysign(std::numeric_limits<float>::quiet_NaN(), neg ? -1.0f : 1.0f);
  return (float)v;   // exact (at most 11 significant bits, exponent within fp32's range); -0.0 stays -0.0
}

float bf16_to_float(uint16_t w) {
  const uint32_t bits = (uint32_t)w << 16;
  float f;
  std::memcpy(&f, &bits, 4);
  return f;
}

void store_code(void* out, uint64_t j, uint32_t code, const Format& f) {
  if (f.K == 16) ((uint16_t*)out)[j] = (uint16_t)code;
  else ((uint8_t*)out)[j] = (uint8_t)code;
}

bool is_8bit_target(int fmt) { return fmt == FMT_E4M3 || fmt == FMT_E5M2 || fmt == FMT_BINARY8P4; }

bool args_ok(int fmt, int variant, int nbits, Format* f) {
  if (!get_format(fmt, f)) return false;
  if (variant < VAR_RNE || variant > VAR_SRC) return false;
  if (variant != VAR_RNE && (nbits < 1 || nbits > 32)) return false;
  return true;
}

// One fused step of Alg. 1 (quantization-aware training of an 8-bit model with 16-bit updates):
//   w16 <- w8;  u16 <- AdamW update in 16-bit;  w8 <- RoundTo8(w16 + u16), SR applied to that rounding.
// The paper gives no more than the listing and "gradient updates computed in BFloat16" (Sec. IV).
// Reading taken here: the 16-bit format is bf16; every arithmetic operation below is ONE IEEE fp32
// operation (round to nearest even) in the order written; every quantity the listing types as F16
// (the moments, the update u, and the sum w16 + u16) is rounded to bf16 with ties-to-even, so the
// value handed to the 8-bit rounding has bf16 precision (D = 4 excess bits for a precision-4 target,
// the count Sec. IV reasons with).  AdamW as commonly defined (decoupled weight decay):
//   m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;
//   u = -lr ( (m / c1) / (sqrt(v / c2) + eps) + wd w ),  c1 = 1 - b1^t, c2 = 1 - b2^t supplied by the caller.
// A NaN produced anywhere is stored as the positive canonical quiet NaN (NaN signs are not portable).
struct AdamW {
  float lr, beta1, beta2, eps, weight_decay, bias_corr1, bias_corr2;
};

uint16_t to_bf16_rne(float x) {
  Format f;
  get_format(FMT_BF16, &f);
  if (std::isnan(x)) return 0x7FC0u;
  return (uint16_t)round_one(x, f, VAR_RNE, 0, 0);
}

// The 16-bit part of one step for one element: updates both moments in place and returns the bf16
// sum w16 + u16 that is handed to RoundTo8 (as a float).
float adamw_sum16(float w, uint16_t g16, uint16_t* m16, uint16_t* v16, const AdamW& a) {
  const float omb1 = 1.0f - a.beta1, omb2 = 1.0f - a.beta2;
  const float g = bf16_to_float(g16);
  const float m0 = bf16_to_float(*m16), v0 = bf16_to_float(*v16);
  const float m1 = std::fmaf(a.beta1, m0, omb1 * g);
  const float v1 = std::fmaf(a.beta2, v0, omb2 * (g * g));
  const uint16_t mq = to_bf16_rne(m1), vq = to_bf16_rne(v1);
  *m16 = mq;
  *v16 = vq;
  const float mh = bf16_to_float(mq) / a.bias_corr1;
  const float vh = bf16_to_float(vq) / a.bias_corr2;
  const float ratio = mh / (std::sqrt(vh) + a.eps);
  const float u = -a.lr * std::fmaf(a.weight_decay, w, ratio);
  const float u16 = bf16_to_float(to_bf16_rne(u));
  return bf16_to_float(to_bf16_rne(w + u16));   // the F16 sum handed to RoundTo8
}

}  // namespace

extern "C" {

// Philox known-answer access.
void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}

// The N-bit integer element `index` draws from stream (seed, step).
uint64_t oracle_random_bits(uint64_t seed, uint64_t step, uint64_t index, int nbits) {
  return random_bits(seed, step, index, nbits);
}

// One element with an explicit n (for exhaustive enumeration over all 2^N draws).
// Returns the code, or 0xFFFFFFFF on invalid arguments.
uint32_t oracle_round_with_n(float x, int fmt, int variant, int nbits, uint64_t n) {
  Format f;
  if (!args_ok(fmt, variant, nbits, &f)) return 0xFFFFFFFFu;
  return round_one(x, f, variant, nbits, n);
}

// Eq. (1) value of a code (NaN / inf per format).
double oracle_decode(uint32_t code, int fmt) {
  Format f;
  if (!get_format(fmt, &f)) return std::numeric_limits<double>::quiet_NaN();
  return decode(code, f);
}

// Target ulp at x: 2^(e~ - P + 1) with e~ of Eq. (2); 1.0 for non-finite x.
double oracle_ulp(float x, int fmt) {
  Format f;
  if (!get_format(fmt, &f)) return std::numeric_limits<double>::quiet_NaN();
  const double a = std::fabs((double)x);
  if (!std::isfinite(a)) return 1.0;
  return std::ldexp(1.0, rounding_exponent(a, f) - f.P + 1);
}

// For each x[k]: the number of draws n in [0, 2^N) whose result differs from the draw-free
// round-down code (i.e. how many draws round away from zero).  Plain enumeration, used by the
// exhaustive-expectation pins.
int oracle_count_up(const float* x, uint64_t count, int fmt, int variant, int nbits, uint64_t* ups) {
  Format f;
  if (!args_ok(fmt, variant, nbits, &f) || variant == VAR_RNE || nbits > 24) return 1;
  for (uint64_t k = 0; k < count; ++k) {
    // n = 0 under SRFF never rounds a non-representable value up (delta < 1): the floor code.
    const uint32_t down = round_one(x[k], f, VAR_SRFF, nbits, 0);
    uint64_t c = 0;
    for (uint64_t n = 0; n < (1ull << nbits); ++n)
      if (round_one(x[k], f, variant, nbits, n) != down) ++c;
    ups[k] = c;
  }
  return 0;
}

// out[j] = FBSR(x[j]) with the bits of global element offset + j, stream (seed, 0).
// out is uint16 codes for bf16, uint8 codes for the fp8 formats.  0 = ok.
int oracle_round(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits,
                 uint64_t seed, uint64_t offset) {
  Format f;
  if (!args_ok(fmt, variant, nbits, &f)) return 1;
  for (uint64_t j = 0; j < n; ++j) {
    const uint64_t r = variant == VAR_RNE ? 0 : random_bits(seed, 0, offset + j, nbits);
    store_code(out, j, round_one(x[j], f, variant, nbits, r), f);
  }
  return 0;
}

// The same, cut into `nthreads` contiguous index ranges (legal because the bits of an
// element depend only on its global index).  Used by the benchmark's CPU-baseline leg.
int oracle_round_threads(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits,
                         uint64_t seed, uint64_t offset, int nthreads) {
  Format f;
  if (!args_ok(fmt, variant, nbits, &f) || nthreads < 1) return 1;
  std::vector<std::thread> pool;
  const uint64_t per = (n + (uint64_t)nthreads - 1) / (uint64_t)nthreads;
  const uint64_t osize = f.K / 8;
  for (int t = 0; t < nthreads; ++t) {
    const uint64_t lo = per * (uint64_t)t;
    if (lo >= n) break;
    const uint64_t cnt = (lo + per <= n) ? per : n - lo;
    pool.emplace_back([=]() {
      oracle_round(x + lo, (char*)out + lo * osize, cnt, fmt, variant, nbits, seed, offset + lo);
    });
  }
  for (auto& th : pool) th.join();
  return 0;
}

// Narrow-source rounding (Sec. III-E: inputs of precision Q = P + D with few excess bits D, e.g.
// bf16 -> E5M2 has D = 5; Fig. 2): the 16-bit source value is taken exactly and rounded as in
// oracle_round.  x: n codes of src_fmt (0 = bf16, 1 = IEEE binary16); fmt: E4M3 or E5M2.
int oracle_round_from16(const uint16_t* x, void* out, uint64_t n, int src_fmt, int fmt, int variant,
                        int nbits, uint64_t seed, uint64_t offset) {
  Format f;
  if (!args_ok(fmt, variant, nbits, &f)) return 1;
  if ((src_fmt != SRC_BF16 && src_fmt != SRC_FP16) || !is_8bit_target(fmt)) return 1;
  for (uint64_t j = 0; j < n; ++j) {
    const uint64_t r = variant == VAR_RNE ? 0 : random_bits(seed, 0, offset + j, nbits);
    store_code(out, j, round_one(widen16(x[j], src_fmt), f, variant, nbits, r), f);
  }
  return 0;
}

// The fp32 bit pattern of widen16 (for pinning the widening against a library view).
uint32_t oracle_widen16(uint16_t code, int src_fmt) {
  const float v = widen16(code, src_fmt);
  uint32_t bits;
  std::memcpy(&bits, &v, 4);
  return bits;
}

// Block-scaled target (Sec. I-A: "blocks of low-precision values are accompanied by a scale factor,
// which may be a power of two"; the paper fixes no rule for choosing it).  Reading taken: blocks of 32
// consecutive elements of the call share the power-of-two scale 2^s with
//   s = clamp(floor(log2 amax) - emax, -127, 127),  amax = max |x| over the block,
//   emax = floor(log2 M) of the element format (8 for E4M3, 15 for E5M2, 7 for binary8p4),
// stored as the byte s + 127 (a pure-exponent code; 0xFF marks a block that holds a NaN or an
// infinity, all of whose elements become the positive canonical NaN), and every element is
// FBSR(x 2^-s) -- an exact scaling -- with the random bits of global index offset + j as in
// oracle_round.  The block's largest element lands in [2^emax, 2^(emax+1)); what exceeds M there is
// rounded by the out-of-range rule.  A block of zeros takes s = -127.  The last block may be short.
int oracle_round_block_scaled(const float* x, uint8_t* out, uint8_t* scales, uint64_t n, int fmt, int variant,
                              int nbits, uint64_t seed, uint64_t offset) {
  Format f;
  if (!args_ok(fmt, variant, nbits, &f) || !is_8bit_target(fmt)) return 1;
  const int emax = std::ilogb(f.M);
  const uint64_t B = 32;
  for (uint64_t b0 = 0; b0 < n; b0 += B) {
    const uint64_t len = n - b0 < B ? n - b0 : B;
    double amax = 0.0;
    bool special = false;
    for (uint64_t k = 0; k < len; ++k) {
      const double a = std::fabs((double)x[b0 + k]);
      if (!std::isfinite(a)) special = true;
      else if (a > amax) amax = a;
    }
    if (special) {
      scales[b0 / B] = 0xFFu;
      for (uint64_t k = 0; k < len; ++k) out[b0 + k] = (uint8_t)f.nan_code;
      continue;
    }
    int s = amax == 0.0 ? -127 : std::ilogb(amax) - emax;
    s = s < -127 ? -127 : (s > 127 ? 127 : s);
    scales[b0 / B] = (uint8_t)(s + 127);
    for (uint64_t k = 0; k < len; ++k) {
      const uint64_t j = b0 + k;
      const uint64_t r = variant == VAR_RNE ? 0 : random_bits(seed, 0, offset + j, nbits);
      out[j] = (uint8_t)round_one(std::ldexp((double)x[j], -s), f, variant, nbits, r);
    }
  }
  return 0;
}

// Alg. 1's "w <- RoundTo(w + u)" in the SGD form u = -lr * g: the bf16 weight is
// widened exactly, the update is one fused multiply-add in fp32 (a single rounding),
// and the fp32 result is rounded back to bf16 with the bits of (seed, step, offset + j).
int oracle_sgd_update(uint16_t* w, const float* g, uint64_t n, float lr, int variant, int nbits,
                      uint64_t seed, uint64_t step, uint64_t offset) {
  Format f;
  if (!args_ok(FMT_BF16, variant, nbits, &f)) return 1;
  for (uint64_t j = 0; j < n; ++j) {
    const float x = std::fmaf(-lr, g[j], bf16_to_float(w[j]));
    const uint64_t r = variant == VAR_RNE ? 0 : random_bits(seed, step, offset + j, nbits);
    w[j] = (uint16_t)round_one(x, f, variant, nbits, r);
  }
  return 0;
}

// w8: n fp8 codes of fmt (E4M3 or E5M2), updated in place; g16: n bf16 gradients; m16, v16: n bf16
// moments, updated in place; p: 7 floats {lr, beta1, beta2, eps, weight_decay, 1 - beta1^t, 1 - beta2^t}.
// Random bits of element j: stream (seed, step), global index offset + j.
int oracle_qat_adamw_step(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t n, int fmt,
                          const float* p, int variant, int nbits, uint64_t seed, uint64_t step, uint64_t offset) {
  Format f;
  if (!args_ok(fmt, variant, nbits, &f) || !is_8bit_target(fmt)) return 1;
  const AdamW a = {p[0], p[1], p[2], p[3], p[4], p[5], p[6]};
  for (uint64_t j = 0; j < n; ++j) {
    const float w = (float)decode(w8[j], f);            // w16 <- w8 (exact)
    const float s16 = adamw_sum16(w, g16[j], &m16[j], &v16[j], a);
    uint32_t code;
    if (std::isnan(s16)) {
      code = f.nan_code;
    } else {
      const uint64_t r = variant == VAR_RNE ? 0 : random_bits(seed, step, offset + j, nbits);
      code = round_one(s16, f, variant, nbits, r);
    }
    w8[j] = (uint8_t)code;
  }
  return 0;
}

// The same step with the 8-bit weights in a generic format (desc as in oracle_round_format8; Sec. IV
// trains in P3109 binary8p4) and any of the seven variants.  A weight code that decodes to NaN (or to
// an unused encoding) enters the arithmetic as NaN.  A NaN sum is stored as the descriptor's NaN code
// without a sign, or as +M when the format has none.
int oracle_qat_adamw_step_format8(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t n,
                                  const int32_t* desc, const float* p, int variant, int nbits, uint64_t seed,
                                  uint64_t step, uint64_t offset) {
  Format8 g;
  if (!get_format8(desc, &g) || !variant8_ok(variant, nbits)) return 1;
  const AdamW a = {p[0], p[1], p[2], p[3], p[4], p[5], p[6]};
  for (uint64_t j = 0; j < n; ++j) {
    const float w = (float)decode8(w8[j], g);           // w16 <- w8 (exact: at most 7 significant bits)
    const float s16 = adamw_sum16(w, g16[j], &m16[j], &v16[j], a);
    uint32_t code;
    if (std::isnan(s16)) {
      code = g.nan_code >= 0 ? (uint32_t)g.nan_code : (uint32_t)g.max_code;
    } else {
      const uint64_t r = variant_draws(variant) ? random_bits(seed, step, offset + j, nbits) : 0;
      code = round_one8(s16, g, variant, nbits, r);
    }
    w8[j] = (uint8_t)code;
  }
  return 0;
}

// Per-bin statistics of the rounding error (the reduction behind Figs. 1 and 2: the mean of
// the rounded samples per input bin, and the bias = mean of (rounded - input) in target
// ulps).  Element j has global index i = offset + j and bin floor(i / group) - first_bin.
// stats is nbins x 4 doubles {count, sum y, sum e, sum e^2}, ACCUMULATED into, where
// y = decoded rounded value and e = (y - x) / ulp_t(x), ulp_t(x) = 2^(e~ - P + 1).
// Non-finite y or x propagate through the sums by IEEE rules.  out may be null.
// Returns 0 ok, 1 bad arguments, 3 an element falls outside [0, nbins).
int oracle_bias_stats(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits,
                      uint64_t seed, uint64_t offset, uint64_t group, uint64_t first_bin,
                      uint32_t nbins, double* stats) {
  Format f;
  if (!args_ok(fmt, variant, nbits, &f) || group == 0) return 1;
  if (n > 0) {
    const uint64_t lo = offset / group, hi = (offset + n - 1) / group;
    if (lo < first_bin || hi - first_bin >= nbins) return 3;
  }
  for (uint64_t j = 0; j < n; ++j) {
    const uint64_t i = offset + j;
    const uint64_t bin = i / group - first_bin;
    const uint64_t r = variant == VAR_RNE ? 0 : random_bits(seed, 0, i, nbits);
    const uint32_t code = round_one(x[j], f, variant, nbits, r);
    if (out) store_code(out, j, code, f);
    const double y = decode(code, f);
    const double e = (y - (double)x[j]) / oracle_ulp(x[j], fmt);
    double* s = stats + 4 * bin;
    s[0] += 1.0;
    s[1] += y;
    s[2] += e;
    s[3] += e * e;
  }
  return 0;
}

// ------------------------------------------------------------ generic formats ---
// desc = {K, P, B, max_code, inf_code, nan_code, nan_signed, neg_zero} (see Format8).
// variant: 0 RNE, 1 SRFF, 2 SRF, 3 SRC (inner ties-to-even), 4 SRC (inner ties-to-odd),
// 5 nearest ties-to-odd, 6 nearest ties-away (0, 5 and 6 draw no bits).

// 0 when the descriptor is acceptable.
int oracle_format8_check(const int32_t* desc) {
  Format8 g;
  return get_format8(desc, &g) ? 0 : 1;
}

// Eq. (1) value of a code under the descriptor (NaN for NaN and unused encodings).
double oracle_decode_format8(uint32_t code, const int32_t* desc) {
  Format8 g;
  if (!get_format8(desc, &g)) return std::numeric_limits<double>::quiet_NaN();
  return decode8(code, g);
}

// The same three with codes of up to 16 bits (K <= 16).
int oracle_format16_check(const int32_t* desc) {
  Format8 g;
  return get_format8(desc, &g, 16) ? 0 : 1;
}

double oracle_decode_format16(uint32_t code, const int32_t* desc) {
  Format8 g;
  if (!get_format8(desc, &g, 16)) return std::numeric_limits<double>::quiet_NaN();
  return decode8(code, g);
}

uint32_t oracle_round_format16_with_n(float x, const int32_t* desc, int variant, int nbits, uint64_t n) {
  Format8 g;
  if (!get_format8(desc, &g, 16) || !variant8_ok(variant, nbits)) return 0xFFFFFFFFu;
  return round_one8(x, g, variant, nbits, n);
}

// oracle_round_format8 for a format of up to 16 bits: out holds one code per 16-bit word (the bits above K zero).
int oracle_round_format16(const void* x, int src, uint16_t* out, uint64_t n, const int32_t* desc, int variant,
                          int nbits, uint64_t seed, uint64_t offset) {
  Format8 g;
  if (!get_format8(desc, &g, 16) || !variant8_ok(variant, nbits) || src < 0 || src > 2) return 1;
  for (uint64_t j = 0; j < n; ++j) {
    const float v = src == 2 ? ((const float*)x)[j] : widen16(((const uint16_t*)x)[j], src);
    const uint64_t r = variant_draws(variant) ? random_bits(seed, 0, offset + j, nbits) : 0;
    out[j] = (uint16_t)round_one8(v, g, variant, nbits, r);
  }
  return 0;
}

// One element with an explicit n.  Returns the code, or 0xFFFFFFFF on invalid arguments.
uint32_t oracle_round_format8_with_n(float x, const int32_t* desc, int variant, int nbits, uint64_t n) {
  Format8 g;
  if (!get_format8(desc, &g) || !variant8_ok(variant, nbits)) return 0xFFFFFFFFu;
  return round_one8(x, g, variant, nbits, n);
}

// x: n values of the source type src (0 = bf16 codes, 1 = IEEE binary16 codes, 2 = fp32); out: n
// bytes, one code each (the bits above K are zero).  Random bits of element j: stream (seed, 0),
// global index offset + j.  Returns 0, or 1 on invalid arguments.
int oracle_round_format8(const void* x, int src, uint8_t* out, uint64_t n, const int32_t* desc, int variant,
                         int nbits, uint64_t seed, uint64_t offset) {
  Format8 g;
  if (!get_format8(desc, &g) || !variant8_ok(variant, nbits) || src < 0 || src > 2) return 1;
  for (uint64_t j = 0; j < n; ++j) {
    const float v = src == 2 ? ((const float*)x)[j] : widen16(((const uint16_t*)x)[j], src);
    const uint64_t r = variant_draws(variant) ? random_bits(seed, 0, offset + j, nbits) : 0;
    out[j] = (uint8_t)round_one8(v, g, variant, nbits, r);
  }
  return 0;
}

// The statistics of oracle_bias_stats for a format given by its descriptor (fp32 inputs): per bin
// {count, sum y, sum e, sum e^2} with y the Eq. (1) value of the rounded code under the descriptor and
// e = (y - x) / ulp_t(x), ulp_t(x) = 2^(e~ - P + 1), e~ of Eq. (2) with the descriptor's B and no upper clamp;
// ulp_t of a non-finite x is 1, as there.  out (one code per byte) may be null.
// Returns 0 ok, 1 bad arguments, 3 an element falls outside [0, nbins).
int oracle_bias_stats_format8(const float* x, uint8_t* out, uint64_t n, const int32_t* desc, int variant, int nbits,
                              uint64_t seed, uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins,
                              double* stats) {
  Format8 g;
  if (!get_format8(desc, &g) || !variant8_ok(variant, nbits) || group == 0) return 1;
  if (n > 0) {
    const uint64_t lo = offset / group, hi = (offset + n - 1) / group;
    if (lo < first_bin || hi - first_bin >= nbins) return 3;
  }
  for (uint64_t j = 0; j < n; ++j) {
    const uint64_t i = offset + j;
    const uint64_t bin = i / group - first_bin;
    const uint64_t r = variant_draws(variant) ? random_bits(seed, 0, i, nbits) : 0;
    const uint32_t code = round_one8(x[j], g, variant, nbits, r);
    if (out) out[j] = (uint8_t)code;
    const double y = decode8(code, g);
    const double a = std::fabs((double)x[j]);
    const double ulp = std::isfinite(a) ? std::ldexp(1.0, rounding_exponent(a, g.f) - g.f.P + 1) : 1.0;
    const double e = (y - (double)x[j]) / ulp;
    double* s = stats + 4 * bin;
    s[0] += 1.0;
    s[1] += y;
    s[2] += e;
    s[3] += e * e;
  }
  return 0;
}

}  // extern "C"
