// fbsr_device.h -- device-side building blocks for few-bit stochastic rounding on gfx950.
//
// Everything here works on the fp32 BIT PATTERN in a fixed-point "code space":
// a 32-bit word whose top bits are the target format's magnitude code and whose low FRAC
// bits are the fraction of one target ulp (the paper's delta, Sec. II-A Eq. (5), scaled by
// 2^FRAC).  In that space every rounding predicate of the paper is one integer addition
// followed by dropping the low FRAC bits (the "addition" implementation the paper mentions
// at the end of Sec. II-A):
//     SRFF  delta + n 2^-N >= 1            ->  + (n << (FRAC - N))
//     SRF   delta + (n + 1/2) 2^-N >= 1    ->  + (n << (FRAC - N)) + (1 << (FRAC - N - 1))
//     SRC   SRFF(RN_even(delta 2^N) 2^-N)  ->  + (2^(FRAC-N-1) - 1) + bit_(FRAC-N)  + (n << (FRAC - N))
//     RNE   ties to even                   ->  SRC with N = 0, n = 0
// A carry out of the fraction increments the significand and, when that overflows, the
// exponent (Sec. II-A: "incrementing the exponent if sigma = 2^P") with no extra work.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fbsr {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Streaming 16-byte load of four consecutive floats (16-byte aligned), read once.
__device__ __forceinline__ f32x4 load_stream4(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
}

enum : int { kBF16 = 0, kE4M3 = 1, kE5M2 = 2, kP4 = 3 };   // kP4: IEEE WG P3109 binary8p4
enum : int { kRNE = 0, kSRFF = 1, kSRF = 2, kSRC = 3 };
enum : int { kSrcBF16 = 0, kSrcFP16 = 1, kSrcFP32 = 2 };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Exact fp32 pattern of a 16-bit source code.
template <int SRC>
__device__ __forceinline__ uint32_t widen16(uint32_t code16) {
  if constexpr (SRC == kSrcBF16) {
    return code16 << 16;
  } else {
    return __float_as_uint(__half2float(__ushort_as_half((unsigned short)code16)));   // v_cvt_f32_f16: exact
  }
}

// ------------------------------------------------------------------------------ Philox ---
// Philox4x32-10 (Salmon et al., SC'11).  Counter (c0..c3), key (k0,k1); the key and the two
// high counter words are wave-uniform, so their arithmetic lands on the scalar unit.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&o)[4]) {
  constexpr uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
  constexpr uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t pa = (uint64_t)MUL_A * c0;
    const uint64_t pb = (uint64_t)MUL_B * c2;
    const uint32_t t0 = (uint32_t)(pb >> 32) ^ c1 ^ (k0 + WEYL_A * (uint32_t)r);
    const uint32_t t2 = (uint32_t)(pa >> 32) ^ c3 ^ (k1 + WEYL_B * (uint32_t)r);
    c1 = (uint32_t)pb;
    c3 = (uint32_t)pa;
    c0 = t0;
    c2 = t2;
  }
  o[0] = c0; o[1] = c1; o[2] = c2; o[3] = c3;
}

// The block with index `blk` of stream (seed, step).
__device__ __forceinline__ void philox_block(uint64_t blk, uint64_t seed, uint64_t step, uint32_t (&o)[4]) {
  philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step, (uint32_t)(step >> 32),
                (uint32_t)seed, (uint32_t)(seed >> 32), o);
}

// ------------------------------------------------------------------------- code spaces ---
// FRAC      fraction bits below the code's last place
// U_MAXFIN  fp32 pattern of M, the largest finite value (Sec. II)
// NAN_FX    canonical quiet NaN, already shifted into code space
template <int FMT> struct Fx;

template <> struct Fx<kBF16> {
  static constexpr int FRAC = 16;
  static constexpr int P = 8, B = 127;
  static constexpr uint32_t U_MAXFIN = 0x7F7F0000u;
  static constexpr uint32_t U_UNCHECKED = U_MAXFIN;   // the largest pattern the unchecked paths accept
  static constexpr uint32_t NAN_FX = 0x7FC00000u;
  static constexpr bool kIsFp8 = false;
  typedef uint16_t code_t;
};

// fp8: FRAC = 24.  A target-normal |x| maps to ((u - (Q << 23)) << S) with Q = 127 - B the
// exponent re-bias and S = FRAC - (24 - P); a target-subnormal |x| (u < U_SUB) maps to
// trunc(|x| * SUB_SCALE), its position on the fixed subnormal grid (Eq. (2) clamps the
// exponent at 1 - B).  Patterns above U_CLAMP are clamped to it first.
template <> struct Fx<kE4M3> {
  static constexpr int FRAC = 24;
  static constexpr int P = 4, B = 7;
  static constexpr uint32_t Q = 120, S = 4;
  static constexpr uint32_t U_MAXFIN = 0x43E00000u;   // 448
  static constexpr uint32_t U_CLAMP = 0x43E00000u;    // saturating: everything above acts as M
  static constexpr uint32_t U_SUB = 121u << 23;       // 2^-6, smallest normal
  static constexpr float SUB_SCALE = 0x1p33f;         // 1 / (2^-9 subnormal spacing) * 2^FRAC
  static constexpr bool kDetRegion = false;
  static constexpr uint32_t DET_ADD = 0;
  static constexpr uint32_t U_UNCHECKED = 0x7F800000u;   // every non-NaN pattern
  static constexpr uint32_t NAN_FX = 0x7F000000u;
  static constexpr uint32_t INF_CODE = 0x100u;        // none
  static constexpr bool kIsFp8 = true;
  typedef uint8_t code_t;
};

template <> struct Fx<kE5M2> {
  static constexpr int FRAC = 24;
  static constexpr int P = 3, B = 15;
  static constexpr uint32_t Q = 112, S = 3;
  static constexpr uint32_t U_MAXFIN = 0x47600000u;   // 57344
  static constexpr uint32_t U_CLAMP = 0x47700000u;    // 61440 = M + ulp(M)/2: maps to code 123.5
  static constexpr uint32_t U_SUB = 113u << 23;       // 2^-14
  static constexpr float SUB_SCALE = 0x1p40f;         // 1 / 2^-16 * 2^FRAC
  static constexpr bool kDetRegion = true;            // (M, 61440): nearest is M; >= 61440: inf
  static constexpr uint32_t DET_ADD = 1u << 23;       // one half: M's significand is odd, the tie goes up
  static constexpr uint32_t U_UNCHECKED = 0x7F800000u;
  static constexpr uint32_t NAN_FX = 0x7E000000u;
  static constexpr uint32_t INF_CODE = 0x7Cu;
  static constexpr bool kIsFp8 = true;
  typedef uint8_t code_t;
};

// IEEE WG P3109 binary8p4 (the format Sec. IV trains in): the value set of OCP E4M3 scaled by one half
// (bias 8 instead of 7, M = 224 at the same code 0x7E), but with infinities at 0x7F / 0xFF, one NaN at
// 0x80 and no negative zero.  Above M the clamp is M + 3/4 ulp(M) and the addend the nearest-even one
// for an even significand (224 = 14 * 16), so the tie 232 stays at M and everything above carries into
// 0x7F.  The NaN code is the sign bit alone, which is what NAN_FX | sign gives for either sign.
template <> struct Fx<kP4> {
  static constexpr int FRAC = 24;
  static constexpr int P = 4, B = 8;
  static constexpr uint32_t Q = 119, S = 4;
  static constexpr uint32_t U_MAXFIN = 0x43600000u;   // 224
  static constexpr uint32_t U_CLAMP = 0x436C0000u;    // 236 = M + 3/4 ulp(M): maps to code 126.75
  static constexpr uint32_t U_SUB = 120u << 23;       // 2^-7, smallest normal
  static constexpr float SUB_SCALE = 0x1p34f;         // 1 / (2^-10 subnormal spacing) * 2^FRAC
  static constexpr bool kDetRegion = true;
  static constexpr uint32_t DET_ADD = (1u << 23) - 1u;
  static constexpr uint32_t U_UNCHECKED = 0x7F800000u;
  static constexpr uint32_t NAN_FX = 0x80000000u;
  static constexpr uint32_t INF_CODE = 0x7Fu;
  static constexpr bool kIsFp8 = true;
  typedef uint8_t code_t;
};

// Wave-uniform shift amounts and constants derived from N once per kernel.
struct Addends {
  uint32_t nbits;      // N (0 for RNE)
  uint32_t shift;      // FRAC - N: position of n's last place
  uint32_t fixed;      // SRF: half of n's last place; SRC/RNE: half of it minus one; SRFF: 0
  uint32_t tie_mask;   // SRC/RNE: 1 when the inner rounding really drops bits, else 0
};

template <int FMT, int VAR>
__device__ __forceinline__ Addends make_addends(int nbits) {
  constexpr int FRAC = Fx<FMT>::FRAC;
  Addends a;
  a.nbits = VAR == kRNE ? 0u : (uint32_t)nbits;
  a.shift = (uint32_t)FRAC - a.nbits;
  a.fixed = 0;
  a.tie_mask = 0;
  if (VAR == kSRF) a.fixed = a.shift >= 1 ? (1u << (a.shift - 1)) : 0u;
  if (VAR == kSRC || VAR == kRNE) {
    // Round(delta 2^N) drops `shift` bits; with shift == 0 it is the identity.
    a.fixed = a.shift >= 1 ? (1u << (a.shift - 1)) - 1u : 0u;
    a.tie_mask = a.shift >= 1 ? 1u : 0u;
  }
  return a;
}

// |x| in code space (see the file header): the magnitude code in the top bits, delta 2^FRAC in
// the low FRAC bits.  For SRC / RNE the bits a target-subnormal input loses to the truncation are
// folded into bit 0 (a sticky bit: it lies below the tie position of the inner rounding).
template <int FMT, int VAR>
__device__ __forceinline__ uint32_t to_code_space(uint32_t bits) {
  typedef Fx<FMT> F;
  const uint32_t u = bits & 0x7FFFFFFFu;
  if constexpr (!F::kIsFp8) {
    return u;   // bf16 shares fp32's exponent range: the pattern already is the code space
  } else {
    const uint32_t uc = u < F::U_CLAMP ? u : F::U_CLAMP;
    const uint32_t normal = (uc << F::S) - (F::Q << (23 + F::S));   // wraps consistently mod 2^32
    const float scaled = fabsf(__uint_as_float(bits)) * F::SUB_SCALE;  // exact: power-of-two scale
    const uint32_t sub = (uint32_t)scaled;                            // truncation toward zero
    const bool is_sub = u < F::U_SUB;
    uint32_t r0 = is_sub ? sub : normal;
    if constexpr (VAR == kSRC || VAR == kRNE) {
      const bool lost = is_sub && ((float)sub != scaled);
      r0 |= lost ? 1u : 0u;
    }
    return r0;
  }
}

// The rounding add in code space.  Returns the rounded MAGNITUDE (code in the top bits, garbage
// below); n < 2^N is the element's random integer (0 for RNE).
// CHECKED = false may be used only when the caller has established that the pattern is not a
// NaN and, for bf16, not above M (those cases take a few extra selects).
template <int FMT, int VAR, bool CHECKED>
__device__ __forceinline__ uint32_t round_magnitude(uint32_t bits, uint32_t r0, uint32_t n, const Addends& a) {
  typedef Fx<FMT> F;
  const uint32_t u = bits & 0x7FFFFFFFu;
  uint32_t add = n << a.shift;
  if constexpr (VAR == kSRF) add += a.fixed;
  if constexpr (VAR == kSRC || VAR == kRNE) add += a.fixed + ((r0 >> a.shift) & a.tie_mask);
  // |x| > M: no randomness, round to nearest even on the unbounded grid (Sec. II): the addend is
  // one half where M's significand is odd (the tie goes up), one half minus one last place where it is even.
  if constexpr (F::kIsFp8) {
    if constexpr (F::kDetRegion) add = u > F::U_MAXFIN ? F::DET_ADD : add;
  } else if constexpr (CHECKED) {
    add = u > F::U_MAXFIN ? (1u << (F::FRAC - 1)) : add;
  }
  uint32_t r = r0 + add;
  if constexpr (CHECKED) r = u > 0x7F800000u ? F::NAN_FX : r;
  return r;
}

// The rounded magnitude with the sign of the source pattern.
template <int FMT>
__device__ __forceinline__ uint32_t with_sign(uint32_t mag, uint32_t bits) {
  if constexpr (FMT == kP4) {
    // no negative zero: a zero magnitude drops the sign (the NaN code, bit 31 alone, passes unchanged)
    return (mag & 0x7F000000u) != 0u ? (mag | (bits & 0x80000000u)) : mag;
  } else {
    return mag | (bits & 0x80000000u);
  }
}

// Rounds one fp32 pattern.  Returns the signed code in the top (32 - FRAC) bits; the low FRAC
// bits are garbage.
template <int FMT, int VAR, bool CHECKED>
__device__ __forceinline__ uint32_t round_pattern(uint32_t bits, uint32_t n, const Addends& a) {
  return with_sign<FMT>(round_magnitude<FMT, VAR, CHECKED>(bits, to_code_space<FMT, VAR>(bits), n, a), bits);
}

// ------------------------------------------------------------ more than 16 random bits ---
// N = 17 .. 24.  |x| / (spacing of the target around x) as a whole part (the magnitude code) and 32 fraction bits,
// plus a sticky bit for what lies below them.  A target-normal |x| drops at most 21 bits, so its fraction is exact;
// a target-subnormal |x| sits on a fixed grid (Eq. (2) clamps the exponent) and may reach far below it, which is
// where the 24-bit code space of the main path would be too short for an addend this fine.
struct WideCode {
  uint32_t whole, frac;
  bool sticky;
};

// u = |pattern| of a finite value, rebias = (127 - B) << 23, p = P, u_sub = pattern of 2^(1-B), bp = B + P.
__device__ __forceinline__ WideCode wide_code(uint32_t u, uint32_t rebias, uint32_t p, uint32_t u_sub, int bp) {
  WideCode c;
  c.sticky = false;
  if (u >= u_sub) {
    const uint32_t r0 = (u - rebias) << p;   // code in the top 8 bits, 24 fraction bits (wraps consistently mod 2^32)
    c.whole = r0 >> 24;
    c.frac = r0 << 8;
  } else {
    const uint32_t field = u >> 23;
    const uint32_t m = field != 0u ? ((u & 0x007FFFFFu) | 0x00800000u) : u;   // fp32 subnormals carry no hidden one
    const int sh = (int)(field != 0u ? field : 1u) + bp - 120;   // |x| / 2^(2-B-P) * 2^32 = m 2^sh; sh <= 7 + P here
    uint64_t r = 0;
    if (sh >= 0) {
      r = (uint64_t)m << sh;
    } else if (sh > -25) {
      r = m >> (-sh);
      c.sticky = (m & ((1u << (-sh)) - 1u)) != 0u;
    } else {
      c.sticky = m != 0u;
    }
    c.whole = (uint32_t)(r >> 32);
    c.frac = (uint32_t)r;
  }
  return c;
}

// 1 when the variant rounds up.  srf: add the half of Eq. (SRF); src: the inner round-to-nearest of Eq. (7), its ties
// to even (tie_xor = 0) or odd (1) in the last of the N kept fraction bits.  17 <= N <= 24, n < 2^N.
__device__ __forceinline__ uint32_t wide_round_up(const WideCode& c, uint32_t n, uint32_t N, bool srf, bool src, uint32_t tie_xor) {
  if (src) {
    const uint32_t drop = 32u - N;   // 8 .. 15
    const uint32_t h = c.frac >> drop, rem = c.frac & ((1u << drop) - 1u), half = 1u << (drop - 1u);
    const bool inc = rem > half || (rem == half && (c.sticky || ((h & 1u) ^ tie_xor) != 0u));
    return (h + (inc ? 1u : 0u) + n) >> N;   // Round(delta 2^N) + n >= 2^N
  }
  // below the lowest addend bit nothing can carry, so neither the low fraction bits nor the sticky bit matter
  const uint64_t add = ((uint64_t)n << (32u - N)) + (srf ? (uint64_t)(1u << (31u - N)) : 0u);
  return (uint32_t)(((uint64_t)c.frac + add) >> 32);
}

// round_pattern for N = 17 .. 24 (the per-element kernels; any pattern).
template <int FMT, int VAR>
__device__ __forceinline__ uint32_t round_pattern_wide(uint32_t bits, uint32_t n, uint32_t N) {
  typedef Fx<FMT> F;
  static_assert(VAR != kRNE, "nearest-even draws no bits");
  if constexpr (!F::kIsFp8) {
    // bf16 drops D = 16 bits, all of them within 16 fraction bits: with N >= D every variant is exact SR on the
    // top D bits of n (App. A-C), which is what the addends of N = 16 compute
    return round_pattern<FMT, VAR, true>(bits, n >> (N - 16u), make_addends<FMT, VAR>(16));
  } else {
    const uint32_t u = bits & 0x7FFFFFFFu;
    // |x| > M or NaN: no randomness enters (Sec. II), any N gives the same code
    if (u > F::U_MAXFIN) return round_pattern<FMT, VAR, true>(bits, 0u, make_addends<FMT, VAR>(1));
    const WideCode c = wide_code(u, F::Q << 23, (uint32_t)F::S, F::U_SUB, F::B + F::P);
    const uint32_t up = wide_round_up(c, n, N, VAR == kSRF, VAR == kSRC, 0u);
    return with_sign<FMT>((c.whole + up) << 24, bits);
  }
}

// The same rounding for N = 17 .. 24 in the 24-bit code space of the main path (the tile kernels; any pattern).  A
// target-normal |x| is exact there, and so is the addend n << (24 - N).  A target-subnormal |x| may lose bits to the
// truncation, all of them below the code space's last place; an addend made of whole last places cannot carry out of
// them, which settles SRFF for every N and SRF up to N = 23.  What is left takes the subnormal position from a float
// product of its own (exact: a power-of-two scale) in units of the random grid, delta~ 2^N plus the whole part:
//   SRF, N = 24   floor(pos + 1/2) = (trunc(2 pos) + 1) >> 1, as  pos + n + 1/2 >= k  <=>  floor(pos + 1/2) + n >= k;
//   SRC           Round(pos) of Eq. (7) is the hardware's round-to-nearest-even of that product.
struct ManyAddends {
  Addends a;          // for N itself: shift = 24 - N, fixed and tie_mask 0 where the shift is 0
  float grid_scale;   // SUB_SCALE 2^-shift: a target-subnormal |x| times this is its position on the random grid
};

template <int FMT, int VAR>
__device__ __forceinline__ ManyAddends make_many_addends(int nbits) {
  ManyAddends w;
  if constexpr (Fx<FMT>::kIsFp8) {
    w.a = make_addends<FMT, VAR>(nbits);
    w.grid_scale = __builtin_amdgcn_ldexpf(Fx<FMT>::SUB_SCALE, -(int)w.a.shift);
  } else {
    w.a = make_addends<FMT, VAR>(16);   // bf16: see round_pattern_wide
    w.grid_scale = 0.0f;
  }
  return w;
}

template <int FMT, int VAR, bool CHECKED>
__device__ __forceinline__ uint32_t round_pattern_many(uint32_t bits, uint32_t n, uint32_t N, const ManyAddends& w) {
  typedef Fx<FMT> F;
  static_assert(VAR != kRNE, "nearest-even draws no bits");
  if constexpr (!F::kIsFp8) {
    return round_pattern<FMT, VAR, CHECKED>(bits, n >> (N - 16u), w.a);
  } else {
    const Addends& a = w.a;
    const uint32_t u = bits & 0x7FFFFFFFu;
    const uint32_t uc = u < F::U_CLAMP ? u : F::U_CLAMP;
    const uint32_t normal = (uc << F::S) - (F::Q << (23 + F::S));
    const float ax = fabsf(__uint_as_float(bits));
    uint32_t in_normal = normal, in_sub;
    if constexpr (VAR == kSRFF) {
      in_sub = (uint32_t)(ax * F::SUB_SCALE);
    } else if constexpr (VAR == kSRF) {
      in_normal = normal + a.fixed;
      const float scaled = ax * F::SUB_SCALE;
      if (a.shift == 0u) in_sub = ((uint32_t)(scaled + scaled) + 1u) >> 1;   // uniform over the launch
      else in_sub = (uint32_t)scaled + a.fixed;
    } else {
      in_normal = normal + a.fixed + ((normal >> a.shift) & a.tie_mask);
      in_sub = (uint32_t)rintf(ax * w.grid_scale) << a.shift;
    }
    uint32_t r0 = u < F::U_SUB ? in_sub : in_normal;
    uint32_t add = n << a.shift;
    if constexpr (F::kDetRegion) {
      const bool above = u > F::U_MAXFIN;
      r0 = above ? normal : r0;
      add = above ? F::DET_ADD : add;
    }
    uint32_t r = r0 + add;
    if constexpr (CHECKED) r = u > 0x7F800000u ? F::NAN_FX : r;
    return with_sign<FMT>(r, bits);
  }
}

// True when round_pattern<.., CHECKED = false> is not allowed for this pattern.
template <int FMT>
__device__ __forceinline__ bool needs_checked(uint32_t u_max) {
  return u_max > Fx<FMT>::U_UNCHECKED;
}

constexpr int kWavesPerBlock = 4;
constexpr int kThreads = 64 * kWavesPerBlock;

// ----------------------------------------------------------- workgroup tile geometry ---
// A 256-thread workgroup handles kTileElems = 2048 consecutive elements, 512 per wave, as
// kRows = 2 rows of 256 per wave (lane l owns elements 256 k + 4 l .. + 3 of row k: one fully
// coalesced 16-byte load per row).  Small tiles and many workgroups stream best on this part:
// measured with a plain 4:1 read:write kernel, 2 rows per thread reach 6.5 TB/s where 4 rows
// reach 6.05 and 16 rows 5.8.
// The tile needs 2048 W bits = 16 W Philox blocks; thread t computes block t (t < 16 W), so
// every block is computed exactly once and the RNG cost per element falls with W.  The lane that
// computes a block is not the lane that consumes its bits, so the blocks go through an LDS strip
// laid out as the tile's linear bit string (element e at bit e W).
// (The fp32 rounding kernels take workgroups of 8 such waves, 4096 elements: WgTile's WAVES.)
constexpr int kRows = 2;
constexpr int kWaveElems = kRows * 256;
constexpr int kTileElems = kWavesPerBlock * kWaveElems;

// Which tile a workgroup takes.  Workgroups are handed to the part's 8 XCDs in turn (workgroup b runs on
// XCD b mod 8), each XCD with an L2 and a share of the memory fabric of its own; with the identity map every
// XCD walks the whole tensor with a stride of 8 tiles.  Here the launch is cut into chunks of 8 R tiles,
// R = 2^log2_run, and within a chunk XCD j takes the j-th run of R consecutive tiles: each XCD then streams
// through contiguous memory.  log2_run = 0 is the identity map.
// A bijection of [0, ntiles): whole chunks are permuted within themselves, the tiles after the last whole
// chunk keep their index.  What a tile computes depends on its index alone, so results do not change.
__device__ __forceinline__ uint32_t xcd_tile(uint32_t wg, uint32_t ntiles, uint32_t log2_run) {
  const uint32_t chunk_mask = (8u << log2_run) - 1u;
  if (wg >= (ntiles & ~chunk_mask)) return wg;
  const uint32_t r = wg & chunk_mask;
  return (wg - r) + ((r & 7u) << log2_run) + (r >> 3);
}

// WAVES: waves per workgroup, 512 elements each (most kernels 4; the fp32 rounding kernels 8, see kRoundWaves).
template <int W, int WAVES = kWavesPerBlock> struct WgTile {
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int ELEMS = WAVES * kWaveElems;
  static constexpr int BLOCKS = ELEMS * W / 128;
  static constexpr int PER_THREAD = (BLOCKS + THREADS - 1) / THREADS;
};

template <int W, int WAVES = kWavesPerBlock>
__device__ __forceinline__ void fill_wg_bits(uint4* strip, int tid, uint64_t wg_blk0, uint64_t seed,
                                             uint64_t step) {
#pragma unroll
  for (int i = 0; i < WgTile<W, WAVES>::PER_THREAD; ++i) {
    const int b = tid + WgTile<W, WAVES>::THREADS * i;
    if (b < WgTile<W, WAVES>::BLOCKS) {
      uint32_t o[4];
      philox_block(wg_blk0 + (uint64_t)b, seed, step, o);
      strip[b] = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

// The 4 W random bits of this lane's four elements in row k of its wave, right-aligned in a
// 64-bit word (element j at bits j W).
template <int W>
__device__ __forceinline__ uint64_t read_wg_row_bits(const uint4* strip, int wave, int lane, int k) {
  const unsigned char* base = reinterpret_cast<const unsigned char*>(strip);
  const int e0 = wave * kWaveElems + k * 256 + 4 * lane;   // first element, tile-relative
  if constexpr (W == 16) {
    return *reinterpret_cast<const uint64_t*>(base + e0 * 2);
  } else if constexpr (W == 8) {
    return *reinterpret_cast<const uint32_t*>(base + e0);
  } else if constexpr (W == 4) {
    return *reinterpret_cast<const uint16_t*>(base + e0 / 2);
  } else if constexpr (W == 2) {
    return base[e0 / 4];
  } else {
    return (uint32_t)(base[e0 / 8] >> ((lane & 1) * 4)) & 0xFu;
  }
}

// The random integers of EIGHT consecutive elements starting at tile-relative element e0 (a
// multiple of 8): the 16-bit-source kernels give every lane one 16-byte load of 8 elements.
template <int W>
__device__ __forceinline__ void read_wg_bits8(const uint4* strip, int e0, uint32_t nbits, uint32_t (&n)[8]) {
  const unsigned char* base = reinterpret_cast<const unsigned char*>(strip);
  if constexpr (W == 32) {   // more than 16 random bits: two Philox blocks
    const uint4 q0 = strip[e0 / 4], q1 = strip[e0 / 4 + 1];
    const uint32_t w[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) n[j] = __builtin_amdgcn_ubfe(w[j], 0u, nbits);
  } else if constexpr (W == 16) {
    const uint4 q = *reinterpret_cast<const uint4*>(base + e0 * 2);
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) n[j] = __builtin_amdgcn_ubfe(w[j >> 1], (uint32_t)(16 * (j & 1)), nbits);
  } else if constexpr (W == 8) {
    const uint2 q = *reinterpret_cast<const uint2*>(base + e0);
    const uint32_t w[2] = {q.x, q.y};
#pragma unroll
    for (int j = 0; j < 8; ++j) n[j] = __builtin_amdgcn_ubfe(w[j >> 2], (uint32_t)(8 * (j & 3)), nbits);
  } else {
    uint32_t w;
    if constexpr (W == 4) w = *reinterpret_cast<const uint32_t*>(base + e0 / 2);
    else if constexpr (W == 2) w = *reinterpret_cast<const uint16_t*>(base + e0 / 4);
    else w = base[e0 / 8];
#pragma unroll
    for (int j = 0; j < 8; ++j) n[j] = __builtin_amdgcn_ubfe(w, (uint32_t)(j * W), nbits);
  }
}

// The random integers of this lane's four elements in row k of its wave, for every slot width: with 32-bit slots
// (more than 16 random bits) the row's four slots are one Philox block.
template <int W>
__device__ __forceinline__ void row_draws4(const uint4* strip, int wave, int lane, int k, uint32_t nbits, uint32_t (&n)[4]);

// With more than 16 random bits: true when the bit count passes what the hardware converts apply exactly to every input
// (they add the top D = 24 - P bits of the random operand to the first D bits below the kept ones and drop what lies
// further down: exact for up to D random bits, D - 1 with SRF's half step, on any input; exact for any count on a
// target-normal input, which has no bits further down).  Then a wave may use them only if it holds no non-zero value
// below the target's normal range.
template <int FMT, int VAR>
__device__ __forceinline__ bool hw_needs_normal_inputs(int nbits) {
  return nbits > 24 - Fx<FMT>::P - (VAR == kSRF ? 1 : 0);
}

// For that test: |pattern| - 1, which sends zero to the top of the range.
__device__ __forceinline__ uint32_t magnitude_less_one(uint32_t bits) { return (bits & 0x7FFFFFFFu) - 1u; }

template <int W>
__device__ __forceinline__ uint32_t slot_bits(uint64_t row_bits, int j, uint32_t nbits) {
  if constexpr (W == 16) {
    const uint32_t w = (uint32_t)(row_bits >> (32 * (j >> 1)));
    return __builtin_amdgcn_ubfe(w, (uint32_t)(16 * (j & 1)), nbits);
  } else {
    return __builtin_amdgcn_ubfe((uint32_t)row_bits, (uint32_t)(j * W), nbits);
  }
}

template <int W>
__device__ __forceinline__ void row_draws4(const uint4* strip, int wave, int lane, int k, uint32_t nbits, uint32_t (&n)[4]) {
  if constexpr (W == 32) {
    const uint4 q = strip[(wave * kWaveElems + k * 256 + 4 * lane) / 4];
    n[0] = __builtin_amdgcn_ubfe(q.x, 0u, nbits); n[1] = __builtin_amdgcn_ubfe(q.y, 0u, nbits);
    n[2] = __builtin_amdgcn_ubfe(q.z, 0u, nbits); n[3] = __builtin_amdgcn_ubfe(q.w, 0u, nbits);
  } else {
    const uint64_t rb = read_wg_row_bits<W>(strip, wave, lane, k);
#pragma unroll
    for (int j = 0; j < 4; ++j) n[j] = slot_bits<W>(rb, j, nbits);
  }
}

// ------------------------------------------------- hardware stochastic-rounding converts ---
// gfx950 has v_cvt_sr_fp8_f32 / v_cvt_sr_bf8_f32 (OCP E4M3 / E5M2): they add the TOP bits of a
// 32-bit random operand to the bits the conversion drops (however many those are: target
// subnormals included) and truncate.  Feeding  n << (32 - N)  therefore is SRFF, and
// (n << (32 - N)) | (1 << (31 - N))  is SRF; SRC first rounds |x| to P + N significant bits
// (nearest-even, on the clamped-exponent grid of Eq. (2)) with a magic-constant float add.
// Verified against the CPU oracle on every fp32 pattern; what the instructions do OUTSIDE the
// finite range differs from this library's readings and is steered here:
//   E4M3: above 448 they return NaN  -> the input is clamped to +-448 first (saturation);
//   E5M2: in (M, 65536) they round stochastically between M and inf -> the random operand is
//         replaced by one half, which gives M below 61440 and inf from there on;
//   NaN comes back with the sign bit set -> NaN inputs never reach this path (the caller's
//         wave-uniform check sends them to the integer path).
// binary8p4 uses the E4M3 convert on 2 x (an exact doubling: the two value sets differ by that factor and
// share their codes up to M = 0x7E); the clamp to +-448 turns every |x| > M into 0x7E, whose last bit is
// then set for |x| > 232 (the infinity 0x7F; the tie 232 itself stays at M, whose significand is even);
// a negative zero result loses its sign.
struct HwAddends {
  uint32_t nbits;     // N
  uint32_t shift;     // 32 - N
  uint32_t half;      // SRF: 1 << (31 - N), else 0
  uint32_t grid_exp;  // SRC: (24 - P - N) << 23, the exponent offset of the magic constant
};

template <int FMT, int VAR>
__device__ __forceinline__ HwAddends make_hw_addends(int nbits) {
  HwAddends h;
  h.nbits = (uint32_t)nbits;
  h.shift = 32u - h.nbits;
  h.half = VAR == kSRF ? (1u << (31u - h.nbits)) : 0u;
  h.grid_exp = (uint32_t)(24 - Fx<FMT>::P - nbits) << 23;
  return h;
}

// Four fp32 patterns and their random integers -> four packed fp8 codes (element 0 in the low
// byte).  None of the patterns may be a NaN.
// MANY: nbits may exceed 24 - P, the number of bits a target-normal input drops.  The grid of SRC's inner rounding is
// then finer than some inputs' own last place; those inputs (|x| >= C) already lie on it and must be left alone, because
// the sum |x| + C would round them in a higher binade.
template <int FMT, int VAR, bool MANY = false>
__device__ __forceinline__ uint32_t round4_fp8_hw(const uint32_t (&bits)[4], const uint32_t (&n)[4], const HwAddends& h) {
  typedef Fx<FMT> F;
  static_assert(F::kIsFp8 && VAR != kRNE, "hardware path: fp8 targets, stochastic variants");
  constexpr uint32_t kSubField = FMT == kP4 ? Fx<kE4M3>::U_SUB : F::U_SUB;   // binary8p4 works on 2 x in E4M3 terms
  int packed = 0;
  uint32_t to_inf = 0;   // binary8p4: the last bit of every byte whose |x| lies above the overflow tie
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float x = __uint_as_float(bits[j]);
    uint32_t rnd = (n[j] << h.shift) | h.half;
    if constexpr (FMT == kP4) {
      to_inf |= fabsf(x) > 232.0f ? (1u << (8 * j)) : 0u;
      x = x + x;
    }
    if constexpr (FMT == kE4M3 || FMT == kP4) x = __builtin_amdgcn_fmed3f(x, -448.0f, 448.0f);
    bool over = false;
    if constexpr (FMT == kE5M2) over = fabsf(x) > 57344.0f;
    if constexpr (VAR == kSRC) {
      // C = 2^(e~ + 24 - P - N): adding and subtracting it rounds |x| to a multiple of
      // 2^(e~ - (P - 1) - N), nearest-even (the inner Round of Eq. (7))
      const uint32_t ef = __float_as_uint(x) & 0x7F800000u;   // after the clamp
      const uint32_t c_bits = (ef > kSubField ? ef : kSubField) + h.grid_exp;
      const float c = __uint_as_float(c_bits);
      float t = (fabsf(x) + c) - c;
      if constexpr (MANY) t = fabsf(x) < c ? t : fabsf(x);
      const float pre = __uint_as_float((__float_as_uint(t) & 0x7FFFFFFFu) | (bits[j] & 0x80000000u));
      x = over ? x : pre;
    }
    if constexpr (FMT == kE5M2) rnd = over ? 0x80000000u : rnd;
    if constexpr (FMT == kE4M3 || FMT == kP4) {
      if (j == 0) packed = __builtin_amdgcn_cvt_sr_fp8_f32(x, (int)rnd, packed, 0);
      if (j == 1) packed = __builtin_amdgcn_cvt_sr_fp8_f32(x, (int)rnd, packed, 1);
      if (j == 2) packed = __builtin_amdgcn_cvt_sr_fp8_f32(x, (int)rnd, packed, 2);
      if (j == 3) packed = __builtin_amdgcn_cvt_sr_fp8_f32(x, (int)rnd, packed, 3);
    } else {
      if (j == 0) packed = __builtin_amdgcn_cvt_sr_bf8_f32(x, (int)rnd, packed, 0);
      if (j == 1) packed = __builtin_amdgcn_cvt_sr_bf8_f32(x, (int)rnd, packed, 1);
      if (j == 2) packed = __builtin_amdgcn_cvt_sr_bf8_f32(x, (int)rnd, packed, 2);
      if (j == 3) packed = __builtin_amdgcn_cvt_sr_bf8_f32(x, (int)rnd, packed, 3);
    }
  }
  if constexpr (FMT == kP4) {
    packed |= (int)to_inf;
    // bytes with a zero magnitude lose their sign bit
    const uint32_t m = (uint32_t)packed & 0x7F7F7F7Fu;
    const uint32_t nonzero = ((m + 0x7F7F7F7Fu) | m) & 0x80808080u;   // 0x80 in every byte whose magnitude is not zero
    return (uint32_t)packed & (nonzero | 0x7F7F7F7Fu);
  }
  return (uint32_t)packed;
}

// Exact value of an 8-bit code (Eq. (1)); the hardware decodes agree with it on all 256 OCP codes, and
// binary8p4's finite values are one half of E4M3's at the same code.
template <int FMT>
__device__ __forceinline__ float fp8_code_value(uint32_t code) {
  if constexpr (FMT == kE4M3) {
    return __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
  } else if constexpr (FMT == kE5M2) {
    return __builtin_amdgcn_cvt_f32_bf8((int)code, 0);
  } else {
    const uint32_t c = code & 0xFFu;
    const float finite = 0.5f * __builtin_amdgcn_cvt_f32_fp8((int)c, 0);
    const float inf = __uint_as_float(0x7F800000u | ((c & 0x80u) << 24));
    const float v = (c & 0x7Fu) == 0x7Fu ? inf : finite;
    return c == 0x80u ? __uint_as_float(0x7FC00000u) : v;
  }
}

// ------------------------------------------- rounding with the error in hand (statistics) ---
// In code space the rounding error needs no second look at the value: with r0 = |x| there and r = r0 + addend,
// the rounded magnitude is r with its fraction cleared, so  (r & ~fraction mask) - r0  is, as a plain integer, the
// error (|y| - |x|) / ulp_t(x) of Sec. III in units of 2^-FRAC -- exact whenever r0 is exact, and valid across a
// carry into the next binade (the first value up there continues this binade's grid).
//   FastRound::rs     the signed code in the top (32 - FRAC) bits, zeros below
//   FastRound::e_int  (|y| - |x|) / ulp_t(x) 2^FRAC, in (-2^FRAC, 2^FRAC): e 2^FRAC for x >= 0, its negative for x < 0
// Preconditions (the caller checks them for a whole wave): no NaN and |x| <= M; fp8 with MIXED = false: every |x|
// target-normal (|x| >= 2^(1-B)); fp8 with MIXED = true: additionally any |x| that is zero or >= 2^(2-B-P-FRAC+23),
// the patterns whose position on the subnormal grid has no bits below 2^-FRAC (bf16 needs no such split: its code
// space is the fp32 pattern itself).
struct FastRound {
  uint32_t rs;
  int32_t e_int;
};

// Smallest |pattern| > 0 a MIXED fast path may see.
template <int FMT> struct FastLimits {
  static constexpr uint32_t U_DEEP = (uint32_t)(128 - Fx<FMT>::B - Fx<FMT>::P) << 23;
};

// POSITIVE: the caller knows that no pattern has its sign bit set (then nothing has to be carried over into rs).
// SUB_ONLY (fp8, with MIXED): the caller knows that every |x| lies below 2^(1-B), so the subnormal grid alone places it.
template <int FMT, int VAR, bool MIXED, bool POSITIVE = false, bool SUB_ONLY = false>
__device__ __forceinline__ FastRound round_fast(uint32_t bits, uint32_t n, const Addends& a) {
  typedef Fx<FMT> F;
  constexpr uint32_t kFracMask = (1u << F::FRAC) - 1u;
  uint32_t r0;
  if constexpr (!F::kIsFp8) {
    r0 = bits;   // the sign rides along in bit 31: no carry reaches it while |x| <= M
  } else {
    constexpr uint32_t kRebias = 0u - (F::Q << (23 + F::S));
    if constexpr (MIXED && SUB_ONLY) {
      r0 = (uint32_t)(fabsf(__uint_as_float(bits)) * F::SUB_SCALE);   // below 2^(FRAC + P - 1): no conversion out of range
    } else if constexpr (MIXED) {
      // |x| is split at the smallest normal value 2^(1-B): what lies above it is placed by the re-biased pattern
      // (of max(|x|, 2^(1-B))), what lies below it on the fixed subnormal grid (of min(|x|, 2^(1-B)), a product
      // below 2^32); the position is the sum of the two less the one they both hold at the split point
      const float ax = fabsf(__uint_as_float(bits)), split = __uint_as_float(F::U_SUB);
      constexpr uint32_t kSplit = 1u << (F::FRAC + F::P - 1);
      const uint32_t nrm = (__float_as_uint(fmaxf(ax, split)) << F::S) + (kRebias - kSplit);
      r0 = nrm + (uint32_t)(fminf(ax, split) * F::SUB_SCALE);
    } else {
      r0 = (bits << F::S) + kRebias;
    }
  }
  uint32_t add = n << a.shift;
  if constexpr (VAR == kSRF) add += a.fixed;
  if constexpr (VAR == kSRC || VAR == kRNE) add += a.fixed + ((r0 >> a.shift) & a.tie_mask);
  const uint32_t t = (r0 + add) & ~kFracMask;
  FastRound f;
  f.e_int = (int32_t)(t - r0);
  if constexpr (F::kIsFp8 && !POSITIVE) f.rs = t | (bits & 0x80000000u);
  else f.rs = t;
  return f;
}

// Value of the code FastRound::rs holds (Eq. (1); finite codes only).
template <int FMT>
__device__ __forceinline__ float fast_value(uint32_t rs) {
  if constexpr (FMT == kBF16) return __uint_as_float(rs);
  else if constexpr (FMT == kE5M2) return __builtin_amdgcn_cvt_f32_bf8((int)rs, 3);
  else if constexpr (FMT == kE4M3) return __builtin_amdgcn_cvt_f32_fp8((int)rs, 3);
  else return 0.5f * __builtin_amdgcn_cvt_f32_fp8((int)rs, 3);   // binary8p4: one half of E4M3's value at the same code
}

// ----------------------------------------------------------- generic formats, K <= 8 ---
// A generic target format and a rounding mode, both reduced on the host to the constants the
// code-space arithmetic needs (computed on the host from the caller's descriptor).
struct Fmt8 {
  uint32_t shift_p;     // frac - (24 - P): a target-normal pattern maps to (u - rebias) << shift_p (P when frac = 24)
  uint32_t rebias;      // (127 - B) << 23
  uint32_t u_max;       // fp32 pattern of M
  uint32_t u_clamp;     // |x| is clamped to this pattern: M when saturating, M + 3/4 ulp(M) with an infinity
  uint32_t u_sub;       // fp32 pattern of 2^(1-B), the smallest normal
  float sub_scale;      // 2^(22 + B + P): a target-subnormal |x| maps to trunc(|x| * sub_scale)
  uint32_t det_add;     // the nearest-even addend that applies above M
  uint32_t max_code;    // magnitude code of M
  uint32_t over_code;   // magnitude code that replaces every code above max_code (infinity)
  uint32_t nan_code;    // code of a NaN input before its sign is applied
  uint32_t nan_sign;    // the sign bit if a NaN input keeps its sign, else 0
  uint32_t sign_bit;    // 1 << (K - 1)
  uint32_t sign_shift;  // 32 - K: (pattern >> sign_shift) & sign_bit is the code's sign
  uint32_t sign_carry;  // sign_bit with -0, sign_bit - 1 without: (mag + sign_carry) & sign_bit tells whether a
                        // magnitude code keeps its sign (every code but a zero without -0), as mag < sign_bit
  uint32_t remap_over;  // 1 when over_code is neither max_code nor the code after it, else 0
  uint32_t unit_lsb;    // 1 << 24 when P = 1 (the significand's last place is the implicit one), else 0
  uint32_t frac;        // fraction bits of the code space: 24 for K <= 8; 32 - K for the 16-bit-code entry point
  int32_t sub_exp;      // frac - 2 + B + P: a target-subnormal |x| maps to trunc(|x| * 2^sub_exp)
};

// The value of every byte as a code of the format (Eq. (1); infinities, and NaN for the NaN code and for
// encodings the format leaves unused), computed on the host.
struct Table8 {
  float v[256];
};

struct Mode8 {
  uint32_t nbits;       // N; 0 for the deterministic modes
  uint32_t shift;       // frac - N
  uint32_t fixed;       // the part of the addend that does not depend on the element
  uint32_t tie_xor;     // inner rounding: 0 ties-to-even, 1 ties-to-odd
  bool ties;            // the mode has an inner round-to-nearest (RNE, RNO, both SRC)
  bool srf;             // the mode adds half a step of the random grid (SRF)
};

// A rounded magnitude code above max_code becomes the infinity's.  The clamp of |x| keeps every rounded magnitude at
// or below max_code + 1 (a saturating format's at or below max_code), which is where most formats have their
// infinity: only one that lies elsewhere needs the exchange (uniform over the launch).
__device__ __forceinline__ uint32_t cap8(uint32_t mag, const Fmt8& f) {
  if (f.remap_over != 0u) mag = mag > f.max_code ? f.over_code : mag;
  return mag;
}

// cap8 on four codes behind ONE branch (the empty statement keeps the compiler from turning the branch into
// selects, which would cost every format what only the rare one needs).
__device__ __forceinline__ void cap8x4(uint32_t (&g)[4], const Fmt8& f) {
  if (f.remap_over != 0u) {
    asm volatile("");
#pragma unroll
    for (int j = 0; j < 4; ++j) g[j] = g[j] > f.max_code ? f.over_code : g[j];
  }
}

// From the rounded magnitude code to the output byte: codes above M become the infinity (or M, saturating),
// the sign goes on (a zero keeps it only in formats with -0), a NaN input becomes the NaN code.
template <bool CHECKED>
__device__ __forceinline__ uint32_t signed8(uint32_t capped_mag, uint32_t bits, const Fmt8& f) {
  uint32_t code = capped_mag | ((bits >> f.sign_shift) & (capped_mag + f.sign_carry) & f.sign_bit);
  const uint32_t sgn = (bits >> f.sign_shift) & f.sign_bit;
  if constexpr (CHECKED) code = (bits & 0x7FFFFFFFu) > 0x7F800000u ? (f.nan_code | (sgn & f.nan_sign)) : code;
  return code;
}

template <bool CHECKED>
__device__ __forceinline__ uint32_t finish8(uint32_t mag, uint32_t bits, const Fmt8& f) {
  return signed8<CHECKED>(cap8(mag, f), bits, f);
}

__device__ __forceinline__ uint32_t pack4_bytes(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3) {
  const uint32_t lo = __builtin_amdgcn_perm(c1, c0, 0x0c0c0400u);   // [c0.b0, c1.b0, 0, 0]
  const uint32_t hi = __builtin_amdgcn_perm(c3, c2, 0x04000c0cu);   // [0, 0, c2.b0, c3.b0]
  return lo | hi;
}

// finish8 (less its NaN case) on four bytes at once.  tops: the top bytes of the four source patterns, element 0 in
// the low byte; mags4: the four capped magnitude codes likewise.  Every magnitude code is below the sign bit and the
// carry at most the sign bit, so no byte's sum reaches into the next.
__device__ __forceinline__ uint32_t with_signs4(uint32_t mags4, uint32_t tops, const Fmt8& f) {
  const uint32_t signs = (tops >> (f.sign_shift - 24u)) & (f.sign_bit * 0x01010101u);
  return mags4 | (signs & (mags4 + f.sign_carry * 0x01010101u));
}

// The top bytes of four fp32 patterns, element 0 in the low byte.
__device__ __forceinline__ uint32_t top_bytes4(const uint32_t (&b)[4]) {
  const uint32_t lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0703u);   // [b0.b3, b1.b3, 0, 0]
  const uint32_t hi = __builtin_amdgcn_perm(b[3], b[2], 0x07030c0cu);   // [0, 0, b2.b3, b3.b3]
  return lo | hi;
}

// round8's sum: the code-space pattern of |x| plus the mode's fixed addend, its tie bit and random_part = n << shift,
// or, above M (*above set; no randomness there, Sec. II), plus the nearest-even addend alone.  With random_part = 0 it
// is the part of the sum that the element's random integer does not enter.  The sum stays below 2^32: the pattern is
// below (max_code + 2) 2^frac and the addends together below 2^frac.
// UNIT = false leaves out the one case that only a format with P = 1 under a mode without random bits has (see
// needs_unit8): the four-at-a-time callers branch on it once per four elements rather than pay for it per element.
template <bool TIES, bool WIDE, bool UNIT = true>
__device__ __forceinline__ uint32_t round8_fixed_part(uint32_t bits, const Fmt8& f, const Mode8& m, bool* above,
                                                      uint32_t random_part = 0u) {
  const uint32_t u = bits & 0x7FFFFFFFu;
  const uint32_t uc = u < f.u_clamp ? u : f.u_clamp;
  const uint32_t normal = (uc - f.rebias) << f.shift_p;
  float scaled;   // exact: power-of-two scale (used below 2^(1-B) only)
  if constexpr (WIDE) scaled = __builtin_amdgcn_ldexpf(__uint_as_float(uc), f.sub_exp);
  else scaled = __uint_as_float(uc) * f.sub_scale;
  const uint32_t sub = (uint32_t)scaled;                     // truncation toward zero
  const bool is_sub = u < f.u_sub;
  uint32_t r0 = is_sub ? sub : normal;
  uint32_t add = random_part + m.fixed;
  if constexpr (TIES) {
    // what a target-subnormal input loses to the truncation is folded into bit 0, below the tie position
    const bool lost = is_sub && ((float)sub != scaled);
    r0 |= lost ? 1u : 0u;
    uint32_t parity_of = r0;
    // P = 1 stores no significand bit: a normal value's significand is its implicit one (odd)
    if constexpr (UNIT) {
      if (f.unit_lsb != 0u) parity_of |= is_sub ? 0u : f.unit_lsb;
    }
    add += ((parity_of >> m.shift) & 1u) ^ m.tie_xor;
  }
  *above = u > f.u_max;
  return r0 + (*above ? f.det_add : add);
}

// One source pattern -> the output byte.  n < 2^N is the element's random integer (0 when the mode
// draws none).  CHECKED = false may be used only when the pattern is known not to be a NaN.
// WIDE = false: the code space has 24 fraction bits (K <= 8).  WIDE = true: f.frac of them (32 - K, for codes of up to
// 16 bits), and the subnormal scale, which may pass fp32's range as a factor, is applied to the exponent.
template <bool TIES, bool WIDE = false, bool UNIT = true>
__device__ __forceinline__ uint32_t round8_magnitude(uint32_t bits, uint32_t n, const Fmt8& f, const Mode8& m) {
  bool above;
  const uint32_t sum = round8_fixed_part<TIES, WIDE, UNIT>(bits, f, m, &above, n << m.shift);
  if constexpr (WIDE) return sum >> f.frac;
  else return sum >> 24;
}

// True when the tie bit of the inner rounding is the implicit one of a P = 1 significand: the unit_lsb bit sits at
// the code space's first place above the fraction, which is the tie position only when no random bits are drawn.
__device__ __forceinline__ bool needs_unit8(const Fmt8& f, const Mode8& m) {
  return f.unit_lsb != 0u && m.shift == f.frac;
}

// round8_magnitude on four elements, the P = 1 case behind one branch (the empty statement keeps it a branch).
template <bool TIES, bool WIDE>
__device__ __forceinline__ void round8_magnitudes4(const uint32_t (&b)[4], const uint32_t (&n)[4], const Fmt8& f, const Mode8& m,
                                                   uint32_t (&g)[4]) {
  if (TIES && needs_unit8(f, m)) {
    asm volatile("");
#pragma unroll
    for (int j = 0; j < 4; ++j) g[j] = round8_magnitude<TIES, WIDE, true>(b[j], n[j], f, m);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) g[j] = round8_magnitude<TIES, WIDE, false>(b[j], n[j], f, m);
  }
}

template <bool TIES, bool CHECKED, bool WIDE = false>
__device__ __forceinline__ uint32_t round8(uint32_t bits, uint32_t n, const Fmt8& f, const Mode8& m) {
  return finish8<CHECKED>(round8_magnitude<TIES, WIDE>(bits, n, f, m), bits, f);
}

// round8 for N = 17 .. 24 (the per-element kernel; any pattern): see round_pattern_wide.
__device__ __forceinline__ uint32_t round8_wide(uint32_t bits, uint32_t n, const Fmt8& f, const Mode8& m) {
  const uint32_t u = bits & 0x7FFFFFFFu;
  if (u > f.u_max) return round8<false, true>(bits, 0u, f, m);   // |x| > M or NaN: the addend does not depend on the mode
  const int bp = (int)(__float_as_uint(f.sub_scale) >> 23) - 127 - 22;   // B + P from sub_scale = 2^(22 + B + P)
  const WideCode c = wide_code(u, f.rebias, f.shift_p, f.u_sub, bp);
  const uint32_t up = wide_round_up(c, n, m.nbits, m.srf, m.ties, m.tie_xor);
  return finish8<false>(c.whole + up, bits, f);
}

// round8 for N = 17 .. 24 in the 24-bit code space (the tile kernels; any pattern): see round_pattern_many.
// grid_scale = sub_scale 2^-shift.  Ties to odd in the subnormal range are taken from the remainder of the truncated
// position (exact: the difference of two floats with a common exponent range).
template <bool TIES>
__device__ __forceinline__ uint32_t round8_many_magnitude(uint32_t bits, uint32_t n, const Fmt8& f, const Mode8& m, float grid_scale) {
  const uint32_t u = bits & 0x7FFFFFFFu;
  const uint32_t uc = u < f.u_clamp ? u : f.u_clamp;
  const uint32_t normal = (uc - f.rebias) << f.shift_p;
  const float ax = __uint_as_float(uc);
  uint32_t in_normal, in_sub;
  if constexpr (TIES) {
    const uint32_t tie_mask = m.shift != 0u ? 1u : 0u;   // with no bit dropped the inner rounding is the identity
    in_normal = normal + m.fixed + (((normal >> m.shift) ^ m.tie_xor) & tie_mask);
    const float pos = ax * grid_scale;
    uint32_t h;
    if (m.tie_xor == 0u) {   // uniform over the launch
      h = (uint32_t)rintf(pos);
    } else {
      h = (uint32_t)pos;
      const float rem = pos - (float)h;
      h += (rem > 0.5f || (rem == 0.5f && (h & 1u) == 0u)) ? 1u : 0u;
    }
    in_sub = h << m.shift;
  } else {
    in_normal = normal + m.fixed;
    const float scaled = ax * f.sub_scale;
    if (m.srf && m.shift == 0u) in_sub = ((uint32_t)(scaled + scaled) + 1u) >> 1;   // uniform over the launch
    else in_sub = (uint32_t)scaled + m.fixed;
  }
  const uint32_t r0 = u < f.u_sub ? in_sub : in_normal;
  const uint32_t sum = u > f.u_max ? normal + f.det_add : r0 + (n << m.shift);
  return sum >> 24;
}

// Four 16-bit codes of a generic format as two words (element 0 in the low half of the first).
template <bool TIES>
__device__ __forceinline__ uint2 round4_codes16(const uint32_t (&b)[4], const uint32_t (&n)[4], bool checked, const Fmt8& f,
                                                const Mode8& m) {
  uint32_t c[4];
  round8_magnitudes4<TIES, true>(b, n, f, m, c);
  cap8x4(c, f);
  if (checked) {
#pragma unroll
    for (int j = 0; j < 4; ++j) c[j] = signed8<true>(c[j], b[j], f);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) c[j] = signed8<false>(c[j], b[j], f);
  }
  return make_uint2(c[0] | (c[1] << 16), c[2] | (c[3] << 16));
}

// MANY: more than 16 random bits (grid_scale: see round8_many).
template <bool TIES, bool MANY = false>
__device__ __forceinline__ uint32_t round4_bytes(const uint32_t (&b)[4], const uint32_t (&n)[4], bool checked,
                                                 const Fmt8& f, const Mode8& m, float grid_scale = 0.0f) {
  uint32_t g[4];
  if constexpr (MANY) {
#pragma unroll
    for (int j = 0; j < 4; ++j) g[j] = round8_many_magnitude<TIES>(b[j], n[j], f, m, grid_scale);
  } else {
    round8_magnitudes4<TIES, false>(b, n, f, m, g);
  }
  cap8x4(g, f);
  if (checked) {   // a NaN among the wave's elements: each byte finished by itself
    return pack4_bytes(signed8<true>(g[0], b[0], f), signed8<true>(g[1], b[1], f), signed8<true>(g[2], b[2], f),
                       signed8<true>(g[3], b[3], f));
  }
  return with_signs4(pack4_bytes(g[0], g[1], g[2], g[3]), top_bytes4(b), f);
}

// Random integer of ONE element with global index i (the per-element kernels).
__device__ __forceinline__ uint32_t element_bits(uint64_t i, int log2_per_block, int W, uint32_t nbits,
                                                 uint64_t seed, uint64_t step) {
  const uint64_t blk = i >> log2_per_block;
  const uint32_t slot = (uint32_t)i & ((1u << log2_per_block) - 1u);
  uint32_t o[4];
  philox_block(blk, seed, step, o);
  const uint32_t bit = slot * (uint32_t)W;
  const uint32_t wi = bit >> 5;
  const uint32_t word = wi == 0 ? o[0] : wi == 1 ? o[1] : wi == 2 ? o[2] : o[3];
  return __builtin_amdgcn_ubfe(word, bit & 31u, nbits);
}

// Packs the codes of four rounded patterns (element 0 in the low bits).
template <int FMT>
__device__ __forceinline__ uint32_t pack4_fp8(uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3) {
  // byte 3 of each word is the signed 8-bit code
  const uint32_t lo = __builtin_amdgcn_perm(r1, r0, 0x0c0c0703u);   // [r0.b3, r1.b3, 0, 0]
  const uint32_t hi = __builtin_amdgcn_perm(r3, r2, 0x07030c0cu);   // [0, 0, r2.b3, r3.b3]
  return lo | hi;
}

__device__ __forceinline__ uint32_t pack2_bf16(uint32_t r0, uint32_t r1) {
  return __builtin_amdgcn_perm(r1, r0, 0x07060302u);   // [r0.hi16, r1.hi16]
}

}  // namespace fbsr
