// fbsr_qat.hip -- kernels behind fbsr_qat_adamw_step and fbsr_qat_adamw_step_format8: one fused step
// of Alg. 1 (w16 <- w8; AdamW update in bf16; w8 <- RoundTo8(w16 + u16) with few-bit stochastic
// rounding).  Per element 7 bytes are read (w8, g, m, v) and 5 written (w8, m, v); the arithmetic is a
// fixed sequence of single IEEE fp32 operations (this file is compiled without contraction; the
// divisions and the square root are the correctly rounded ones) so that it can be reproduced bit for bit.
//
// The 8-bit format enters through a codec: how a weight code becomes a value and how the bf16 sum is
// rounded back.  FixedCodec is OCP E4M3 / E5M2 with the hardware decode and the hardware SR converts;
// Codec8 is any (K, P, B; M) with K <= 8 (Sec. II), decoded through a 256-entry table in LDS and rounded
// by the code-space addition of round8.
#include <type_traits>

#include "fbsr_launch.h"

namespace fbsr {

// bf16 code of x rounded to nearest even; any NaN becomes the positive canonical NaN.
__device__ __forceinline__ uint32_t bf16_rne(float x, const Addends& a16) {
  const uint32_t bits = __float_as_uint(x);
  const uint32_t r = round_pattern<kBF16, kRNE, true>(bits, 0u, a16) >> 16;
  return (bits & 0x7FFFFFFFu) > 0x7F800000u ? 0x7FC0u : r;
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two fp32 values -> two bf16 codes (a in the low half), round to nearest even, as one v_cvt_pk_bf16_f32.
// On every non-NaN pattern the instruction equals the integer rounding of bf16_rne (overflow to infinity
// and fp32 subnormals included; checked on all 2^32 patterns); a NaN comes back quieted in place, which is
// not this library's canonical NaN, so callers keep NaNs away from results they store.
__device__ __forceinline__ uint32_t bf16_pair_hw(float a, float b) {
  const f32x2 v = {a, b};
  const bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }

// x / c for a bf16-valued x and a wave-uniform c in [2^-20, 1] with r = 1 / c correctly rounded: one multiply and two
// fused multiply-adds (a residual correction of the quotient) instead of the full division sequence.  The result
// is the correctly rounded quotient, signed zeros included, whenever x is zero or |x| >= 2^-103 -- checked on a
// CPU against the division for all 2^7 bf16 significands times all 2^23 divisor significands, and across the
// exponent range; a quotient that overflows, or an infinite or NaN x, comes back as infinity or NaN, and a NaN
// sends the wave to the exact path anyway.  *tiny is set when |x| is non-zero and below 2^(MIN_EXP - 1), MIN_EXP >= -102.
template <int MIN_EXP>
__device__ __forceinline__ float div_by_uniform(float x, float c, float r, bool* tiny) {
  *tiny = *tiny || __builtin_amdgcn_frexp_expf(x) < MIN_EXP;   // the exponent of a zero reads 0
  const float q = x * r;
  const float t = __fmaf_rn(q, c, -x);   // exact: q c - x
  return __fmaf_rn(-t, r, q);
}

// sqrt(x), correctly rounded, for x that is +-0, +infinity or at least 2^-96 (a negative or NaN x gives a NaN):
// the hardware approximation (within one ulp) moved to a neighbour when the sign of the residual x - s' s, one
// fused multiply-add each, says so.  This is the core of the usual expansion of sqrtf without its rescaling of
// small inputs, which exists to keep these residuals from underflowing; equal to sqrtf on all 1.9 x 10^9 patterns
// of that domain (checked on the device), and checked on a CPU for every starting value within one ulp.
__device__ __forceinline__ float sqrt_not_tiny(float x) {
  const float s = __builtin_amdgcn_sqrtf(x);
  const float lo = __uint_as_float(__float_as_uint(s) - 1u), hi = __uint_as_float(__float_as_uint(s) + 1u);
  const float r_lo = __fmaf_rn(-lo, s, x), r_hi = __fmaf_rn(-hi, s, x);
  float out = r_lo <= 0.0f ? lo : s;
  out = r_hi > 0.0f ? hi : out;
  return out;
}

// The AdamW update u (before its rounding to bf16) from the weight and the new bf16 moments.
__device__ __forceinline__ float qat_update(float w, float mq, float vq, const AdamWScalars& p) {
  const float mh = mq / p.bias_corr1;
  const float vh = vq / p.bias_corr2;
  const float ratio = mh / (sqrtf(vh) + p.eps);
  return -p.lr * __fmaf_rn(p.weight_decay, w, ratio);
}

// n / d, correctly rounded, for a d in [2^-28, 2^65) and an n that is zero, infinite, a NaN or of magnitude at least
// 2^-40: the reciprocal approximation, one Newton step on it, the quotient and two residual corrections of it, then
// v_div_fixup_f32 for the sign of a zero quotient and for an infinite or NaN operand.  These are the operations of the
// full division sequence without its pre-scaling of the operands (v_div_scale_f32, and the rescaling inside
// v_div_fmas_f32), which exists to keep the intermediates of extreme operands in range and changes no bit when they
// are: on this domain no reciprocal, quotient or residual leaves the normal range unless the quotient itself
// overflows, and then the result is the same infinity, or a NaN that sends the wave to the exact path.  A NaN d gives
// a NaN.  Checked on a CPU from every reciprocal start within one ulp (tests/unscaled_division_check.c; the one start
// no such sequence survives -- an all-ones divisor significand with the start below the rounded reciprocal -- is not
// what v_rcp_f32 returns), and on the device against the division itself (fbsr_check_qat_division).
__device__ __forceinline__ float div_in_range(float n, float d) {
  const float r0 = __builtin_amdgcn_rcpf(d);
  const float e = __fmaf_rn(-d, r0, 1.0f);
  const float r = __fmaf_rn(e, r0, r0);
  float q = n * r;
  float rem = __fmaf_rn(-d, q, n);
  q = __fmaf_rn(rem, r, q);
  rem = __fmaf_rn(-d, q, n);
  q = __fmaf_rn(rem, r, q);
  return __builtin_amdgcn_div_fixupf(q, d, n);
}

// sqrt(v / bias_corr2) for a bf16 second moment v by two table reads.  With E the exponent field of v, H = E >> 1 and
// p = E & 1, v = (1.f x 2^(p + 1)) x (2^(H - 64))^2, and both the correctly rounded division by a constant and the
// correctly rounded square root commute with such a scaling while every value stays normal.  So the root is
// roots[p, f] x scales[sign, H] with
//   roots[p, f]   = sqrt((1.f x 2^(p + 1)) / bias_corr2), 256 entries, filled by each workgroup with the two routines above;
//   scales[0, H]  = 2^(H - 64) for 1 <= H <= 116 (v in [2^-125, 2^107): the quotient stays normal for bias_corr2 in [2^-20, 1]);
//   scales[0, 0]  = 0: a v below 2^-125, zero included, has a root below 2^-52, which the sum with an eps of at least
//                   2^-28 (the host checks it) drops entirely, so a zero root gives the same denominator;
//   every other entry (an overflowing quotient, infinity, NaN, any set sign bit) = NaN, which reaches the sum of
//                   weight and update and sends the wave to the exact path.
struct RootTables {
  float roots[256];
  float scales[256];
};

__device__ __forceinline__ void fill_root_tables(RootTables* t, int tid, const AdamWScalars& p) {
  bool unused = false;
  const float x = __uint_as_float(((128u + ((uint32_t)tid >> 7)) << 23) | (((uint32_t)tid & 127u) << 16));
  t->roots[tid] = sqrt_not_tiny(div_by_uniform<-100>(x, p.bias_corr2, p.rcp_corr2, &unused));
  const uint32_t H = (uint32_t)tid;
  t->scales[tid] = __uint_as_float(H == 0u ? 0u : (H <= 116u ? (H + 63u) << 23 : 0x7FC00000u));
}

// HALF 0: the second moment in the low half of `pair`, 1: in the high half.
template <int HALF>
__device__ __forceinline__ float root_of_corrected(const RootTables* t, uint32_t pair) {
  const uint32_t at_root = HALF ? (pair >> 14) & 0x3FCu : (pair << 2) & 0x3FCu;     // byte offsets: (p, f) and (sign, H)
  const uint32_t at_scale = HALF ? (pair >> 22) & 0x3FCu : (pair >> 6) & 0x3FCu;
  const float root = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(t->roots) + at_root);
  const float scale = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(t->scales) + at_scale);
  return root * scale;
}

// The same value as qat_update with the division by bias_corr1 taken by div_by_uniform, the corrected second moment's
// root by root_of_corrected and the last division by div_in_range (the host has checked the scalars' ranges, and
// *tiny sends a first moment below 2^-40 to the exact path).
template <int HALF>
__device__ __forceinline__ float qat_update_fast(float w, float mq, uint32_t v_pair, const AdamWScalars& p, const RootTables* t,
                                                 bool* tiny) {
  const float mh = div_by_uniform<-39>(mq, p.bias_corr1, p.rcp_corr1, tiny);
  const float ratio = div_in_range(mh, root_of_corrected<HALF>(t, v_pair) + p.eps);
  return -p.lr * __fmaf_rn(p.weight_decay, w, ratio);
}

// ------------------------------------------------------------------------------- codecs ---
// A codec provides
//   Args            what the host passes (a kernel argument)
//   kDraws          the rounding consumes random bits
//   kTable          the decode needs the 256-entry table staged in LDS
//   nbits()         N
//   value<J>(lo,hi) value of element J of eight packed codes (main path)
//   value_of(code)  value of one code
//   suspicious(lo, hi)  the eight weight codes hold one that value<J> does not decode
//   must_recompute(sa, sb)  the sums may not go through round4 (a NaN)
//   round4(b, n)    four bf16-valued fp32 patterns, none a NaN -> four packed codes
//   round1(s16, n)  one bf16 code (a NaN is the canonical positive one) -> code
template <int FMT, int VAR>
struct FixedCodec {
  struct Args {
    int nbits;
  };
  static constexpr bool kDraws = VAR != kRNE;
  static constexpr bool kTable = false;
  Addends a8;
  HwAddends hw;
  __device__ FixedCodec(const Args& a, const float*) : a8(make_addends<FMT, VAR>(a.nbits)) {
    hw = HwAddends{0, 0, 0, 0};
    if constexpr (VAR != kRNE) hw = make_hw_addends<FMT, VAR>(a.nbits);
  }
  __device__ __forceinline__ uint32_t nbits() const { return a8.nbits; }
  // the hardware decode agrees with Eq. (1) on all 256 OCP codes; binary8p4's finite values are one half of
  // E4M3's at the same code (its infinities come back as NaN, which sends the wave to value_of, and its NaN
  // 0x80 as -0: see suspicious)
  template <int J>
  __device__ __forceinline__ float value(int lo, int hi) const {
    const int word = J < 4 ? lo : hi;
    if constexpr (FMT == kE4M3) return __builtin_amdgcn_cvt_f32_fp8(word, J & 3);
    else if constexpr (FMT == kP4) return 0.5f * __builtin_amdgcn_cvt_f32_fp8(word, J & 3);
    else return __builtin_amdgcn_cvt_f32_bf8(word, J & 3);
  }
  __device__ __forceinline__ float value_of(uint32_t code) const { return fp8_code_value<FMT>(code); }
  // true when the main path may not be used for these eight weight codes
  __device__ __forceinline__ bool suspicious(uint32_t lo, uint32_t hi) const {
    if constexpr (FMT == kP4) {   // a byte 0x80 (NaN) anywhere
      const uint32_t a = lo ^ 0x80808080u, b = hi ^ 0x80808080u;
      return (((a - 0x01010101u) & ~a) | ((b - 0x01010101u) & ~b)) & 0x80808080u;
    } else {
      return false;
    }
  }
  // true when the pair of sums may not go through round4: a NaN
  __device__ __forceinline__ bool must_recompute(float sa, float sb) const { return __builtin_isunordered(sa, sb); }
  __device__ __forceinline__ uint32_t round4(const uint32_t (&b)[4], const uint32_t (&n)[4]) const {
    if constexpr (VAR != kRNE) {
      return round4_fp8_hw<FMT, VAR>(b, n, hw);
    } else {
      return pack4_fp8<FMT>(round_pattern<FMT, kRNE, false>(b[0], 0u, a8), round_pattern<FMT, kRNE, false>(b[1], 0u, a8),
                            round_pattern<FMT, kRNE, false>(b[2], 0u, a8), round_pattern<FMT, kRNE, false>(b[3], 0u, a8));
    }
  }
  __device__ __forceinline__ uint32_t round1(uint32_t s16, uint32_t n) const {
    const uint32_t r = round_pattern<FMT, VAR, true>(s16 << 16, n, a8) >> Fx<FMT>::FRAC;
    return s16 == 0x7FC0u ? (Fx<FMT>::NAN_FX >> Fx<FMT>::FRAC) : r;
  }
};

template <bool TIES, bool DRAWS>
struct Codec8 {
  struct Args {
    Fmt8 f;
    Mode8 m;
    Table8 t;
  };
  static constexpr bool kDraws = DRAWS;
  static constexpr bool kTable = true;
  Fmt8 f;
  Mode8 m;
  const float* table;   // LDS
  __device__ Codec8(const Args& a, const float* lds_table) : f(a.f), m(a.m), table(lds_table) {}
  __device__ __forceinline__ uint32_t nbits() const { return m.nbits; }
  template <int J>
  __device__ __forceinline__ float value(int lo, int hi) const {
    const uint32_t word = (uint32_t)(J < 4 ? lo : hi);
    return table[(word >> (8 * (J & 3))) & 0xFFu];
  }
  __device__ __forceinline__ float value_of(uint32_t code) const { return table[code & 0xFFu]; }
  __device__ __forceinline__ bool suspicious(uint32_t, uint32_t) const { return false; }
  __device__ __forceinline__ bool must_recompute(float sa, float sb) const { return __builtin_isunordered(sa, sb); }
  __device__ __forceinline__ uint32_t round4(const uint32_t (&b)[4], const uint32_t (&n)[4]) const {
    return round4_bytes<TIES>(b, n, false, f, m);
  }
  // a NaN sum (the canonical positive NaN) becomes the NaN code without a sign, or +M in a format without NaN
  __device__ __forceinline__ uint32_t round1(uint32_t s16, uint32_t n) const { return round8<TIES, true>(s16 << 16, n, f, m); }
};

struct QatOut {
  uint32_t w8, m16, v16;
};

// One element, every rounding on the integer path (canonical NaNs): the per-element kernel and any wave
// of the tile kernel that meets a NaN.
template <class CODEC>
__device__ __forceinline__ QatOut qat_one(const CODEC& c, uint32_t w8, uint32_t g16, uint32_t m16, uint32_t v16, uint32_t n,
                                          const AdamWScalars& p, float omb1, float omb2, const Addends& a16) {
  const float w = c.value_of(w8);
  const float g = __uint_as_float(g16 << 16);
  const float m0 = __uint_as_float(m16 << 16), v0 = __uint_as_float(v16 << 16);
  const float m1 = __fmaf_rn(p.beta1, m0, omb1 * g);
  const float v1 = __fmaf_rn(p.beta2, v0, omb2 * (g * g));
  QatOut o;
  o.m16 = bf16_rne(m1, a16);
  o.v16 = bf16_rne(v1, a16);
  const float u = qat_update(w, __uint_as_float(o.m16 << 16), __uint_as_float(o.v16 << 16), p);
  const float u16 = __uint_as_float(bf16_rne(u, a16) << 16);
  const uint32_t s16 = bf16_rne(w + u16, a16);
  o.w8 = c.round1(s16, n);
  return o;
}

// One workgroup per 2048-element tile, 8 consecutive elements per lane: one 8-byte load of weights,
// three 16-byte loads (gradient, both moments), the same back minus the gradient.  Elements are worked
// on in pairs so that every bf16 rounding is half a packed hardware convert and the moments leave in
// their storage layout.  A NaN anywhere in the wave's sums sends the wave through qat_one instead.
template <class CODEC, int W>
__global__ __launch_bounds__(kThreads) void qat_tiles(uint8_t* __restrict__ w8, const uint16_t* __restrict__ g16,
                                                      uint16_t* __restrict__ m16, uint16_t* __restrict__ v16,
                                                      AdamWScalars p, typename CODEC::Args ca, uint64_t seed, uint64_t step,
                                                      uint64_t blk0, uint32_t xcd_lg) {
  typedef WgTile<W> T;
  __shared__ uint4 strip[T::BLOCKS];
  __shared__ float table[CODEC::kTable ? 256 : 1];
  __shared__ RootTables roots;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int e0 = wave * kWaveElems + 8 * lane;
  const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x, xcd_lg);
  const uint64_t g0 = (uint64_t)tile * T::ELEMS + (uint64_t)e0;
  const uint64_t wq = *reinterpret_cast<const uint64_t*>(w8 + g0);
  const u32x4 gq = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(g16 + g0));
  const u32x4 mq = *reinterpret_cast<const u32x4*>(m16 + g0);
  const u32x4 vq = *reinterpret_cast<const u32x4*>(v16 + g0);
  if constexpr (CODEC::kTable) table[threadIdx.x] = ca.t.v[threadIdx.x];
  if constexpr (CODEC::kDraws) fill_wg_bits<W>(strip, threadIdx.x, blk0 + (uint64_t)tile * T::BLOCKS, seed, step);
  if (p.fast_div != 0) fill_root_tables(&roots, threadIdx.x, p);   // uniform over the launch
  __syncthreads();
  const CODEC c(ca, table);
  const Addends a16 = make_addends<kBF16, kRNE>(0);
  const float omb1 = 1.0f - p.beta1, omb2 = 1.0f - p.beta2;
  uint32_t n[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if constexpr (CODEC::kDraws) read_wg_bits8<W>(strip, e0, c.nbits(), n);
  const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w}, mw[4] = {mq.x, mq.y, mq.z, mq.w}, vw[4] = {vq.x, vq.y, vq.z, vq.w};
  const int wlo = (int)(uint32_t)wq, whi = (int)(uint32_t)(wq >> 32);
  uint32_t mo[4], vo[4], so[4];
  bool nan_seen = c.suspicious((uint32_t)wlo, (uint32_t)whi);   // also set for anything else the main path does not take
  auto do_pair = [&](auto hc, auto fast_tag) {   // elements 2h (low halves) and 2h + 1 (high halves)
    constexpr int h = decltype(hc)::value;
    constexpr bool FAST = decltype(fast_tag)::value;
    const float wa = c.template value<2 * h>(wlo, whi), wb = c.template value<2 * h + 1>(wlo, whi);
    const float ga = bf16_lo(gw[h]), gb = bf16_hi(gw[h]);
    const float m1a = __fmaf_rn(p.beta1, bf16_lo(mw[h]), omb1 * ga), m1b = __fmaf_rn(p.beta1, bf16_hi(mw[h]), omb1 * gb);
    const float v1a = __fmaf_rn(p.beta2, bf16_lo(vw[h]), omb2 * (ga * ga)), v1b = __fmaf_rn(p.beta2, bf16_hi(vw[h]), omb2 * (gb * gb));
    mo[h] = bf16_pair_hw(m1a, m1b);
    vo[h] = bf16_pair_hw(v1a, v1b);
    uint32_t uo;
    if constexpr (FAST) {
      uo = bf16_pair_hw(qat_update_fast<0>(wa, bf16_lo(mo[h]), vo[h], p, &roots, &nan_seen),
                        qat_update_fast<1>(wb, bf16_hi(mo[h]), vo[h], p, &roots, &nan_seen));
    } else {
      uo = bf16_pair_hw(qat_update(wa, bf16_lo(mo[h]), bf16_lo(vo[h]), p), qat_update(wb, bf16_hi(mo[h]), bf16_hi(vo[h]), p));
    }
    const float sa = wa + bf16_lo(uo), sb = wb + bf16_hi(uo);
    nan_seen = nan_seen || c.must_recompute(sa, sb);   // a NaN weight, moment or update always reaches the sum
    so[h] = bf16_pair_hw(sa, sb);
  };
  if (p.fast_div != 0) {   // uniform over the launch
    do_pair(std::integral_constant<int, 0>{}, std::true_type{});
    do_pair(std::integral_constant<int, 1>{}, std::true_type{});
    do_pair(std::integral_constant<int, 2>{}, std::true_type{});
    do_pair(std::integral_constant<int, 3>{}, std::true_type{});
  } else {
    do_pair(std::integral_constant<int, 0>{}, std::false_type{});
    do_pair(std::integral_constant<int, 1>{}, std::false_type{});
    do_pair(std::integral_constant<int, 2>{}, std::false_type{});
    do_pair(std::integral_constant<int, 3>{}, std::false_type{});
  }
  uint64_t wo = 0;
  if (__any(nan_seen)) {
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      mo[h] = 0;
      vo[h] = 0;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int sh = 16 * (j & 1);
      const QatOut o = qat_one(c, (uint32_t)(wq >> (8 * j)) & 0xFFu, (gw[j >> 1] >> sh) & 0xFFFFu, (mw[j >> 1] >> sh) & 0xFFFFu,
                               (vw[j >> 1] >> sh) & 0xFFFFu, n[j], p, omb1, omb2, a16);
      mo[j >> 1] |= o.m16 << sh;
      vo[j >> 1] |= o.v16 << sh;
      wo |= (uint64_t)o.w8 << (8 * j);
    }
  } else {
    uint32_t packed[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const uint32_t b4[4] = {so[2 * q] << 16, so[2 * q] & 0xFFFF0000u, so[2 * q + 1] << 16, so[2 * q + 1] & 0xFFFF0000u};
      const uint32_t n4[4] = {n[4 * q], n[4 * q + 1], n[4 * q + 2], n[4 * q + 3]};
      packed[q] = c.round4(b4, n4);
    }
    wo = (uint64_t)packed[0] | ((uint64_t)packed[1] << 32);
  }
  *reinterpret_cast<uint64_t*>(w8 + g0) = wo;
  u32x4 t;
  t.x = mo[0]; t.y = mo[1]; t.z = mo[2]; t.w = mo[3];
  *reinterpret_cast<u32x4*>(m16 + g0) = t;
  t.x = vo[0]; t.y = vo[1]; t.z = vo[2]; t.w = vo[3];
  *reinterpret_cast<u32x4*>(v16 + g0) = t;
}

// Measurement aid: the tile kernel's loads and stores with the arithmetic taken out (each output word is the input
// word combined with the gradient's by one exclusive or): 7 bytes read and 5 written per element in the same
// launch shape.  What this reaches is the practical ceiling of the fused step's traffic on the part at hand.
__global__ __launch_bounds__(kThreads) void stream75_tiles(uint8_t* __restrict__ w8, const uint16_t* __restrict__ g16,
                                                           uint16_t* __restrict__ m16, uint16_t* __restrict__ v16, uint32_t xcd_lg) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x, xcd_lg);
  const uint64_t g0 = (uint64_t)tile * kTileElems + (uint64_t)(wave * kWaveElems + 8 * lane);
  const uint64_t wq = *reinterpret_cast<const uint64_t*>(w8 + g0);
  const u32x4 gq = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(g16 + g0));
  u32x4 mq = *reinterpret_cast<const u32x4*>(m16 + g0);
  u32x4 vq = *reinterpret_cast<const u32x4*>(v16 + g0);
  mq.x ^= gq.x; mq.y ^= gq.y; mq.z ^= gq.z; mq.w ^= gq.w;
  vq.x ^= gq.w; vq.y ^= gq.z; vq.z ^= gq.y; vq.w ^= gq.x;
  *reinterpret_cast<uint64_t*>(w8 + g0) = wq ^ (uint64_t)(gq.x & 0x01010101u);
  *reinterpret_cast<u32x4*>(m16 + g0) = mq;
  *reinterpret_cast<u32x4*>(v16 + g0) = vq;
}

// Device self-checks of the two identities the tile kernel's update arithmetic rests on (the same device functions,
// run on the part at hand): counts[0] counts the operand pairs for which div_in_range differs from the division
// (a NaN from div_in_range counts as agreement: the tile kernel then recomputes), counts[1] the second-moment codes
// for which the tabulated root differs from sqrtf(v / bias_corr2) (a NaN from the table likewise).
__global__ __launch_bounds__(kThreads) void check_division(const float* __restrict__ num, const float* __restrict__ den, uint64_t count,
                                                           unsigned long long* __restrict__ counts) {
  const uint64_t k = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k >= count) return;
  const float n = num[k], d = den[k];
  const float got = div_in_range(n, d), want = n / d;
  if (got == got && __float_as_uint(got) != __float_as_uint(want)) atomicAdd(counts, 1ull);
}

__global__ __launch_bounds__(kThreads) void check_corrected_root(AdamWScalars p, unsigned long long* __restrict__ counts) {
  __shared__ RootTables roots;
  fill_root_tables(&roots, threadIdx.x, p);
  __syncthreads();
  const uint32_t pair = ((uint32_t)blockIdx.x << 8 | threadIdx.x) * 0x00010001u;   // the same code in both halves
  const float v = bf16_hi(pair);
  const float want = sqrtf(v / p.bias_corr2);
  const float lo = root_of_corrected<0>(&roots, pair), hi = root_of_corrected<1>(&roots, pair);
  const bool tiny = (pair & 0x7F800000u) < 0x01000000u;   // exponent field 0 or 1: the table reads zero, the root is below 2^-52
  const bool ok_lo = lo != lo || (tiny ? (lo == 0.0f && want < 0x1p-52f) : __float_as_uint(lo) == __float_as_uint(want));
  const bool ok_hi = hi != hi || (tiny ? (hi == 0.0f && want < 0x1p-52f) : __float_as_uint(hi) == __float_as_uint(want));
  if (!ok_lo || !ok_hi) atomicAdd(counts + 1, 1ull);
}

// One thread per element: any alignment, any offset, ragged heads and tails.
template <class CODEC>
__global__ __launch_bounds__(kThreads) void qat_elems(uint8_t* __restrict__ w8, const uint16_t* __restrict__ g16,
                                                      uint16_t* __restrict__ m16, uint16_t* __restrict__ v16, uint64_t n,
                                                      AdamWScalars p, typename CODEC::Args ca, int W, int log2_per_block,
                                                      uint64_t seed, uint64_t step, uint64_t offset) {
  __shared__ float table[CODEC::kTable ? 256 : 1];
  if constexpr (CODEC::kTable) {
    table[threadIdx.x] = ca.t.v[threadIdx.x];
    __syncthreads();
  }
  const uint64_t j = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (j >= n) return;
  const CODEC c(ca, table);
  const Addends a16 = make_addends<kBF16, kRNE>(0);
  uint32_t rnd = 0;
  if constexpr (CODEC::kDraws) rnd = element_bits(offset + j, log2_per_block, W, c.nbits(), seed, step);
  const QatOut o = qat_one(c, w8[j], g16[j], m16[j], v16[j], rnd, p, 1.0f - p.beta1, 1.0f - p.beta2, a16);
  w8[j] = (uint8_t)o.w8;
  m16[j] = (uint16_t)o.m16;
  v16[j] = (uint16_t)o.v16;
}

namespace {

template <class CODEC>
hipError_t launch_tiles_w(int W, uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t ntiles,
                          const AdamWScalars& p, const typename CODEC::Args& ca, uint64_t seed, uint64_t step, uint64_t blk0,
                          hipStream_t stream) {
  const dim3 grid((unsigned)ntiles), block(kThreads);
#define FBSR_QAT_LAUNCH(WW) \
  hipLaunchKernelGGL((qat_tiles<CODEC, WW>), grid, block, 0, stream, w8, g16, m16, v16, p, ca, seed, step, blk0, kXcdLgQat)
  if constexpr (!CODEC::kDraws) {
    FBSR_QAT_LAUNCH(8);
  } else {
    switch (W) {
      case 1: FBSR_QAT_LAUNCH(1); break;
      case 2: FBSR_QAT_LAUNCH(2); break;
      case 4: FBSR_QAT_LAUNCH(4); break;
      case 8: FBSR_QAT_LAUNCH(8); break;
      default: FBSR_QAT_LAUNCH(16); break;
    }
  }
#undef FBSR_QAT_LAUNCH
  return hipGetLastError();
}

// nbits: N of a mode that draws bits (unused otherwise).
template <class CODEC>
hipError_t run(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t n, const AdamWScalars& p,
               const typename CODEC::Args& ca, int nbits, uint64_t seed, uint64_t step, uint64_t offset, hipStream_t stream) {
  const int W = CODEC::kDraws ? slot_width(nbits) : 8;
  Split s = split_range(n, offset, W, !CODEC::kDraws, reinterpret_cast<uintptr_t>(g16), 2, 16,
                        reinterpret_cast<uintptr_t>(w8), 1, 8, reinterpret_cast<uintptr_t>(m16), 2, 16);
  if ((reinterpret_cast<uintptr_t>(v16) + s.head * 2) % 16 != 0) {
    s.head = 0;
    s.ntiles = 0;
  }
  return run_split(
      s, n,
      [&](uint64_t first, uint64_t count) {
        hipLaunchKernelGGL((qat_elems<CODEC>), elems_grid(count), dim3(kThreads), 0, stream, w8 + first, g16 + first, m16 + first,
                           v16 + first, count, p, ca, W, log2_of(128 / W), seed, step, offset + first);
        return hipGetLastError();
      },
      [&](uint64_t first, uint64_t count) {
        return launch_tiles_w<CODEC>(W, w8 + first, g16 + first, m16 + first, v16 + first, count, p, ca, seed, step,
                                     (offset + first) / (uint64_t)(128 / W), stream);
      });
}

template <int FMT>
hipError_t run_v(int variant, uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t n,
                 const AdamWScalars& p, int nbits, uint64_t seed, uint64_t step, uint64_t offset, hipStream_t stream) {
  switch (variant) {
    case kRNE: return run<FixedCodec<FMT, kRNE>>(w8, g16, m16, v16, n, p, {nbits}, nbits, seed, step, offset, stream);
    case kSRFF: return run<FixedCodec<FMT, kSRFF>>(w8, g16, m16, v16, n, p, {nbits}, nbits, seed, step, offset, stream);
    case kSRF: return run<FixedCodec<FMT, kSRF>>(w8, g16, m16, v16, n, p, {nbits}, nbits, seed, step, offset, stream);
    default: return run<FixedCodec<FMT, kSRC>>(w8, g16, m16, v16, n, p, {nbits}, nbits, seed, step, offset, stream);
  }
}

}  // namespace

hipError_t launch_check_division(const float* num, const float* den, uint64_t count, unsigned long long* counts, hipStream_t stream) {
  return in_pieces(count, kMaxElemsPerLaunch, [&](uint64_t at, uint64_t m) {
    hipLaunchKernelGGL(check_division, elems_grid(m), dim3(kThreads), 0, stream, num + at, den + at, m, counts);
    return hipGetLastError();
  });
}

hipError_t launch_check_corrected_root(const AdamWScalars& p, unsigned long long* counts, hipStream_t stream) {
  hipLaunchKernelGGL(check_corrected_root, dim3(256), dim3(kThreads), 0, stream, p, counts);
  return hipGetLastError();
}

hipError_t launch_stream75(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t ntiles, hipStream_t stream) {
  return in_pieces(ntiles, kMaxTilesPerLaunch, [&](uint64_t t0, uint64_t count) {
    const uint64_t e0 = t0 * kTileElems;
    hipLaunchKernelGGL(stream75_tiles, dim3((unsigned)count), dim3(kThreads), 0, stream, w8 + e0, g16 + e0, m16 + e0, v16 + e0,
                       kXcdLgQat);
    return hipGetLastError();
  });
}

hipError_t launch_qat_adamw(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t n, int fmt,
                            const AdamWScalars& p, int variant, int nbits, uint64_t seed, uint64_t step,
                            uint64_t offset, hipStream_t stream) {
  if (fmt == kE4M3) return run_v<kE4M3>(variant, w8, g16, m16, v16, n, p, nbits, seed, step, offset, stream);
  if (fmt == kE5M2) return run_v<kE5M2>(variant, w8, g16, m16, v16, n, p, nbits, seed, step, offset, stream);
  return run_v<kP4>(variant, w8, g16, m16, v16, n, p, nbits, seed, step, offset, stream);
}

hipError_t launch_qat_adamw_format8(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t n,
                                    const Fmt8& f, const Mode8& m, const Table8& t, const AdamWScalars& p, uint64_t seed,
                                    uint64_t step, uint64_t offset, hipStream_t stream) {
  const int nbits = (int)m.nbits;
  if (m.nbits != 0) {
    if (m.ties) return run<Codec8<true, true>>(w8, g16, m16, v16, n, p, {f, m, t}, nbits, seed, step, offset, stream);
    return run<Codec8<false, true>>(w8, g16, m16, v16, n, p, {f, m, t}, nbits, seed, step, offset, stream);
  }
  if (m.ties) return run<Codec8<true, false>>(w8, g16, m16, v16, n, p, {f, m, t}, nbits, seed, step, offset, stream);
  return run<Codec8<false, false>>(w8, g16, m16, v16, n, p, {f, m, t}, nbits, seed, step, offset, stream);
}

}  // namespace fbsr
