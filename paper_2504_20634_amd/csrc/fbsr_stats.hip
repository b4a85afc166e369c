// fbsr_stats.hip -- kernels behind fbsr_bias_stats: round as fbsr_round and reduce, per bin,
// {count, sum y, sum e, sum e^2} with y the decoded rounded value and e = (y - x) / ulp_t(x)
// in fp64 -- the measurement behind Figs. 1 and 2 (mean rounded value per input, bias in
// target ulps, Sec. III).  Bins are runs of `group` consecutive global indices.
//
// Reduction order is fixed (lane-local sums -> a fixed tree across the wave -> the four waves' sums
// added in wave order -> for a bin that continues in a neighbouring chunk one record per chunk in the
// workspace, added per bin lane-strided and through the same tree), so results are bit-reproducible;
// no floating-point atomics are used.
#include <mutex>
#include <type_traits>

#include "fbsr_launch.h"
#include "fbsr_stats_common.h"

namespace fbsr {

// Decoded value of the signed code held in the top bits of r (Eq. (1)).  The hardware decodes agree with Eq. (1) on
// every finite fp8 code, give infinities for E5M2's and NaN for the NaN codes (whose sign and payload do not matter
// to a sum).
template <int FMT>
__device__ __forceinline__ float decode_top(uint32_t r) {
  if constexpr (!Fx<FMT>::kIsFp8) return __uint_as_float(r & 0xFFFF0000u);
  else return fp8_code_value<FMT>(r >> 24);
}

// 1 / ulp_t(x) = 2^(P - 1 - e~), e~ = max(floor(log2|x|), 1 - B) (Eq. (2)), built from the
// fp32 exponent field (a field of 0 is below every format's clamp).
template <int FMT>
__device__ __forceinline__ double inv_ulp(uint32_t bits) {
  typedef Fx<FMT> F;
  constexpr uint32_t kMinField = (uint32_t)(1 - F::B + 127) << 23;          // exponent field of the clamp 1 - B
  constexpr uint32_t kTop = (uint32_t)(1023 + F::P - 1 + 127) << 20;        // fp64 exponent of 2^(P-1) re-biased
  const uint32_t ef = bits & 0x7F800000u;
  const uint32_t hi = kTop - ((ef > kMinField ? ef : kMinField) >> 3);      // 2^(P - 1 - e~)
  return __hiloint2double((int)hi, 0);
}

// A lane's share of a span is 64 elements.  64 values of E4M3 (multiples of 2^-9 up to 448) or of binary8p4
// (multiples of 2^-10 up to 224) sum to a multiple of that step below 2^24 steps: exact in fp32 in any order, so
// the sum of y runs there and is widened when the wave closes a bin.
// E4M3 has no infinity: every |x| > M becomes +-M (the library's reading of Sec. II for a saturating format), and the
// error of such an element is a plain integer too.  With |x| = m 2^(e - 23), m the 24-bit significand and e >= 8, and
// ulp_t(x) = 2^(e - 3):  e 2^20 = (M - |x|) / ulp_t(x) 2^20 = (7 << (29 - e)) - m, for e <= 29.
template <int FMT> struct kSaturates { static constexpr bool value = FMT == kE4M3; };
constexpr uint32_t kSaturatedLimit = (uint32_t)(127 + 30) << 23;   // patterns below 2^30

template <int FMT> struct SumYInFp32 { static constexpr bool value = FMT == kE4M3 || FMT == kP4; };

// A lane's running sums for the bin its wave is in.  The integer part serves the elements rounded by round_fast
// (e as an integer multiple of 2^-FRAC: a lane adds at most 64 of them, each below 2^FRAC in magnitude, before its
// wave closes the span, so 32 bits hold their sum and 64 bits the sum of their squares, both exactly); the fp64 part
// serves the elements of the general path.
struct LaneSums {
  int32_t se_i, neg_i;   // sum of e_int ^ s and of s, s = -1 for a negative x and 0 otherwise: their difference is the signed sum
  long long see_i;
  int32_t se20_i;        // the same two sums for the saturated path, whose errors come in units of 2^-20 (signed already)
  long long see20_i;
  float sy32;           // sum y in fp32 for the formats whose 64 values per lane add exactly there
  double sy, se, see;
};

// One workgroup per chunk of kStatsChunkElems consecutive elements, one wave per span of kStatsSpanElems of them,
// walked in pairs of rows of 256 (lane l owns elements 4 l .. 4 l + 3 of a row: one coalesced 16-byte load).  A wave
// draws the random bits of its own span -- lane l computes block 64 k + l of the span in round k, so one round
// serves 8192 / W elements, and the blocks pass through a strip of LDS that only this wave touches -- and keeps
// its sums in registers; where a bin ends inside the span the sums are closed (wave_total) into the wave's row of
// `part`, one entry per bin the chunk touches.  Nothing in the loop waits for another wave: the one barrier of the
// kernel stands after it, in code every thread reaches.  Then the four rows are added in wave order; the chunk's
// first and last bin go to the workspace (they may continue in the neighbouring chunks; stats_finalize adds them
// up), the bins in between are complete and are added to the caller's statistics right here.
//
// Per pair of rows the wave picks, uniformly, the cheapest path the pair's 512 elements allow (see do_pair): one of
// three integer flavours of round_fast with integer error sums, or the general path in fp64.
template <int FMT, int VAR, int W>
__global__ __launch_bounds__(kThreads) void stats_spans(const float* __restrict__ x, void* __restrict__ out,
                                                        uint64_t npairs, int nbits, uint64_t seed, uint64_t blk0,
                                                        uint64_t i0, uint64_t group, uint64_t first_bin,
                                                        uint64_t chunk_base, double* __restrict__ records,
                                                        double* __restrict__ stats) {
  typedef Fx<FMT> F;
  constexpr bool DRAWS = VAR != kRNE;
  constexpr bool MANY = W == 32 && DRAWS;                         // more than 16 bits: a lane's row is one block of its own
  constexpr int PPR = W >= 16 ? 1 : (W >= 2 ? 16 / W : 8);        // pairs of rows one round of 64 blocks serves
  constexpr int SPAN_BLOCKS = kStatsSpanElems / 128 * (W > 16 ? 16 : W);   // blocks that hold the span's bits (W <= 16)
  __shared__ uint4 strips[kWavesPerBlock][2][64];
  __shared__ double part[kWavesPerBlock][kStatsMaxBinsPerChunk][kStatsRecordDoubles];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // in a scalar register: what follows from it is uniform
  const uint64_t chunk = chunk_base + blockIdx.x;
  const uint64_t i_end = i0 + npairs * kStatsPairElems;
  const uint64_t chunk_lo = i0 + chunk * kStatsChunkElems;        // < i_end: the grid has one workgroup per started chunk
  const uint64_t chunk_hi = chunk_lo + kStatsChunkElems < i_end ? chunk_lo + kStatsChunkElems : i_end;
  const uint64_t bin_first = chunk_lo / group;
  const int nbins_here = (int)((chunk_hi - 1) / group - bin_first) + 1;   // <= kStatsMaxBinsPerChunk: group >= kStatsMinGroup

  for (int t = lane; t < nbins_here * (int)kStatsRecordDoubles; t += 64) (&part[wave][0][0])[t] = 0.0;

  const uint64_t span_lo = chunk_lo + (uint64_t)wave * kStatsSpanElems;
  const uint64_t pair0 = chunk * (kStatsChunkElems / kStatsPairElems) + (uint64_t)(wave * kStatsSpanPairs);
  const int my_pairs = pair0 >= npairs ? 0 : (npairs - pair0 < (uint64_t)kStatsSpanPairs ? (int)(npairs - pair0) : kStatsSpanPairs);
  const Addends a = make_addends<FMT, VAR>(MANY ? kMaxTileNbits : nbits);
  const uint64_t span_blk = blk0 + (chunk * (kStatsChunkElems / 128) + (uint64_t)wave * (kStatsSpanElems / 128)) * (uint64_t)W;
  uint4* strip = &strips[wave][0][0];

  // round k of the span's bits into half k & 1 of the wave's strip
  auto draw = [&](int k) {
    if constexpr (DRAWS && !MANY) {
      const int b = k * 64 + lane;
      if (b < SPAN_BLOCKS) {
        uint32_t o[4];
        philox_block(span_blk + (uint64_t)b, seed, 0, o);
        strip[(k & 1) * 64 + lane] = make_uint4(o[0], o[1], o[2], o[3]);
      }
      __builtin_amdgcn_wave_barrier();   // the wave's own LDS traffic keeps program order; this keeps the compiler to it

    }
  };

  LaneSums cur = {0, 0, 0, 0, 0, 0.0f, 0.0, 0.0, 0.0};
  int slot = my_pairs > 0 ? (int)(span_lo / group - bin_first) : 0;
  uint64_t next_bin = my_pairs > 0 ? group - span_lo % group : 0;   // span-relative index at which the next bin starts

  // closes the sums of the bin the wave is in
  auto close_bin = [&]() {
    constexpr double kUnit = 1.0 / (double)((uint64_t)1 << F::FRAC);
    const double t0 = wave_total(cur.sy + (double)cur.sy32);
    constexpr double kUnit20 = 1.0 / (double)(1 << 20);
    double se = cur.se + (double)(cur.se_i - cur.neg_i) * kUnit, see = cur.see + (double)cur.see_i * (kUnit * kUnit);
    if constexpr (kSaturates<FMT>::value) {
      se += (double)cur.se20_i * kUnit20;
      see += (double)cur.see20_i * (kUnit20 * kUnit20);
    }
    const double t1 = wave_total(se);
    const double t2 = wave_total(see);
    if (lane == 0) {
      part[wave][slot][0] = t0; part[wave][slot][1] = t1; part[wave][slot][2] = t2;
    }
    slot += 1;
    cur = {0, 0, 0, 0, 0, 0.0f, 0.0, 0.0, 0.0};
  };

  const float* xs = x + (span_lo - i0);
  f32x4 va[kRows], vb[kRows];
  // exists = false: the pair lies past the span's end; every lane then reads the span's first 16 bytes (a load is
  // issued either way, see below, but one that moves a single cache line instead of the pair's 2 KiB).
  auto load_pair = [&](f32x4 (&v)[kRows], int p, bool exists) {
#pragma unroll
    for (int k = 0; k < kRows; ++k) v[k] = load_stream4(xs + (exists ? p * kStatsPairElems + k * 256 + 4 * lane : 0));
  };

  // Walks the bins of the elements [lo_e, lo_e + len) of the span: add_all() adds all of them to the running sums,
  // add_some(first, last) those whose index relative to lo_e lies in [first, last).
  auto over_bins = [&](int lo_e, int len, auto add_all, auto add_some) {
    const int hi_e = lo_e + len;
    if (next_bin >= (uint64_t)hi_e) {
      add_all();
      return;
    }
    int from = 0;
    while (next_bin < (uint64_t)hi_e) {   // uniform over the wave
      const int cut = (int)next_bin - lo_e;
      add_some(from, cut);
      close_bin();
      from = cut;
      next_bin += group;
    }
    add_some(from, len);
  };

  // The random integers of this lane's four elements in row k of pair p.
  auto row_draws = [&](int p, int k, uint32_t (&n)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) n[j] = 0;
    if constexpr (MANY) {
      uint32_t o[4];
      philox_block(span_blk + (uint64_t)((p * kRows + k) * 64 + lane), seed, 0, o);
#pragma unroll
      for (int j = 0; j < 4; ++j) n[j] = __builtin_amdgcn_ubfe(o[j], 0u, (uint32_t)nbits);
    } else if constexpr (DRAWS) {
      const uint64_t rb = read_row_bits<W>(strip + ((p / PPR) & 1) * 64, (p % PPR) * kStatsPairElems + k * 256 + 4 * lane);
#pragma unroll
      for (int j = 0; j < 4; ++j) n[j] = slot_bits<W>(rb, j, a.nbits);
    }
  };

  // The general path for row k of pair p: the checked rounding, and e = (y - x) / ulp_t(x) with every step in fp64
  // (Sec. III), so that non-finite values follow IEEE arithmetic.  It is rare, and it is kept small rather than
  // fast: one row at a time, its elements read again (from the cache) so that the registers of the fast paths are
  // not held across it.
  auto general_row = [&](int p, int k) {
    const int e0 = p * kStatsPairElems + k * 256;   // span-relative index of the row
    const f32x4 v = *reinterpret_cast<const f32x4*>(xs + (e0 + 4 * lane));
    const uint32_t b[4] = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
    uint32_t n[4], r[4];
    row_draws(p, k, n);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if constexpr (MANY) r[j] = round_pattern_wide<FMT, VAR>(b[j], n[j], (uint32_t)nbits);
      else r[j] = round_pattern<FMT, VAR, true>(b[j], n[j], a);
    }
    if (out != nullptr) {
      const uint64_t row = (span_lo - i0) / 4 + (uint64_t)(e0 / 4 + lane);   // units of 4 elements
      if constexpr (F::kIsFp8)
        reinterpret_cast<uint32_t*>(out)[row] = pack4_fp8<FMT>(r[0], r[1], r[2], r[3]);
      else
        reinterpret_cast<uint64_t*>(out)[row] = (uint64_t)pack2_bf16(r[0], r[1]) | ((uint64_t)pack2_bf16(r[2], r[3]) << 32);
    }
    auto add_one = [&](uint32_t bits, uint32_t rr) {
      const double y = (double)decode_top<FMT>(rr);
      const double e = (y - (double)__uint_as_float(bits)) * inv_ulp<FMT>(bits);
      cur.sy += y;
      cur.se += e;
      cur.see = fma(e, e, cur.see);
    };
    over_bins(
        e0, 256,
        [&]() {
#pragma unroll
          for (int j = 0; j < 4; ++j) add_one(b[j], r[j]);
        },
        [&](int first, int last) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int e = 4 * lane + j;
            if (e >= first && e < last) add_one(b[j], r[j]);
          }
        });
  };

  // everything for pair p of the span, whose elements are in v
  auto do_pair = [&](const f32x4 (&v)[kRows], int p) {
    uint32_t b[kRows][4];
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
      b[k][0] = __float_as_uint(v[k].x); b[k][1] = __float_as_uint(v[k].y);
      b[k][2] = __float_as_uint(v[k].z); b[k][3] = __float_as_uint(v[k].w);
    }
    // Which path: a cascade of wave-uniform tests, the cheapest first.
    //   kPositive  every pattern, taken as an unsigned integer, lies between those of 2^(1-B) (bf16: 0) and M: no sign
    //              bit, no NaN, nothing out of range, (fp8) nothing below the normal range;
    //   kSigned    the same for |x|, either sign;
    //   kMixed     (fp8) as kSigned, with zeros and target-subnormal values that the 24-bit code space places exactly;
    //   kPositiveMixed  (fp8) as kMixed when no pattern has its sign bit set;
    //   kPositiveSubnormal  (fp8) as kPositiveMixed when every value lies below the normal range;
    //   kGeneral   everything else.
    //   kSaturated / kPositiveSaturated  (E4M3) every |x| above M and below 2^30: y = +-M, the error an integer again.
    enum : int { kPositive, kSigned, kMixed, kPositiveMixed, kPositiveSubnormal, kSaturated, kPositiveSaturated, kGeneral };
    int path = kGeneral;
    if constexpr (!MANY) {
      uint32_t top = 0, bottom = 0xFFFFFFFFu;
#pragma unroll
      for (int k = 0; k < kRows; ++k)
#pragma unroll
        for (int j = 0; j < 4; j += 2) {
          top = max(top, max(b[k][j], b[k][j + 1]));
          if constexpr (F::kIsFp8) bottom = min(bottom, min(b[k][j], b[k][j + 1]));
        }
      bool ok;
      if constexpr (F::kIsFp8) ok = !__any(top > F::U_MAXFIN || bottom < F::U_SUB);
      else ok = !__any(top > F::U_MAXFIN);
      bool ok_mixed = false;   // positive, <= M, nothing between zero and the smallest exactly placed pattern (zero itself excluded too)
      if constexpr (F::kIsFp8) ok_mixed = !ok && !__any(top > F::U_MAXFIN || bottom < FastLimits<FMT>::U_DEEP);
      bool ok_saturated = false;
      if constexpr (kSaturates<FMT>::value) ok_saturated = !ok && !ok_mixed && !__any(bottom <= F::U_MAXFIN || top >= kSaturatedLimit);
      if (ok) {
        path = kPositive;
      } else if (ok_mixed) {
        path = kPositiveMixed;
        if constexpr (F::kIsFp8) {
          if (!__any(top >= F::U_SUB)) path = kPositiveSubnormal;
        }
      } else if (ok_saturated) {
        path = kPositiveSaturated;
      } else if constexpr (F::kIsFp8) {
        // (|x| pattern - pattern of 2^(1-B)) * 2 as an unsigned number: small for target-normal |x| <= M, huge otherwise
        uint32_t m = 0;
#pragma unroll
        for (int k = 0; k < kRows; ++k)
#pragma unroll
          for (int j = 0; j < 4; j += 2)
            m = max(m, max((b[k][j] << 1) - 2u * F::U_SUB, (b[k][j + 1] << 1) - 2u * F::U_SUB));
        if (!__any(m > 2u * (F::U_MAXFIN - F::U_SUB))) {
          path = kSigned;
        } else {
          uint32_t hi = 0, lo = 0xFFFFFFFFu;   // largest |pattern|; smallest |pattern| - 1 (zero wraps to the top)
#pragma unroll
          for (int k = 0; k < kRows; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const uint32_t u = b[k][j] & 0x7FFFFFFFu;
              hi = max(hi, u);
              lo = min(lo, u - 1u);
            }
          if (!__any(hi > F::U_MAXFIN || lo < FastLimits<FMT>::U_DEEP - 1u)) path = kMixed;
          if constexpr (kSaturates<FMT>::value) {
            if (!__any(lo < F::U_MAXFIN || hi >= kSaturatedLimit)) path = kSaturated;   // lo = smallest |pattern| - 1
          }
        }
      } else {
        // largest |x|: among the negative patterns the unsigned maximum (top), among the others the signed one
        int32_t mi = 0;
#pragma unroll
        for (int k = 0; k < kRows; ++k)
#pragma unroll
          for (int j = 0; j < 4; j += 2) mi = max(mi, max((int32_t)b[k][j], (int32_t)b[k][j + 1]));
        if (!__any((top & 0x7FFFFFFFu) > F::U_MAXFIN || mi > (int32_t)F::U_MAXFIN)) path = kSigned;
      }
    }
    if (path == kGeneral) {
#pragma unroll 1
      for (int k = 0; k < kRows; ++k) general_row(p, k);
      return;
    }

    // the three integer paths share everything but the flavour of round_fast and the handling of the sign
    auto integer_pair = [&](auto mixed_tag, auto positive_tag, auto sub_only_tag) {
      constexpr bool MIXED = decltype(mixed_tag)::value, POSITIVE = decltype(positive_tag)::value, SUB_ONLY = decltype(sub_only_tag)::value;
      FastRound fr[kRows][4];
#pragma unroll
      for (int k = 0; k < kRows; ++k) {
        uint32_t n[4];
        row_draws(p, k, n);
#pragma unroll
        for (int j = 0; j < 4; ++j) fr[k][j] = round_fast<FMT, VAR, MIXED, POSITIVE, SUB_ONLY>(b[k][j], n[j], a);
      }
      if (out != nullptr) {
        const uint64_t orow = (span_lo - i0) / 4 + (uint64_t)(p * (kStatsPairElems / 4) + lane);   // units of 4 elements
#pragma unroll
        for (int k = 0; k < kRows; ++k) {
          if constexpr (F::kIsFp8) {
            uint32_t packed = pack4_fp8<FMT>(fr[k][0].rs, fr[k][1].rs, fr[k][2].rs, fr[k][3].rs);
            if constexpr (FMT == kP4 && MIXED) {   // no negative zero: a byte with a zero magnitude loses its sign
              const uint32_t mg = packed & 0x7F7F7F7Fu;
              packed &= (((mg + 0x7F7F7F7Fu) | mg) & 0x80808080u) | 0x7F7F7F7Fu;
            }
            reinterpret_cast<uint32_t*>(out)[orow + (uint64_t)(k * 64)] = packed;
          } else {
            reinterpret_cast<uint64_t*>(out)[orow + (uint64_t)(k * 64)] =
                (uint64_t)pack2_bf16(fr[k][0].rs, fr[k][1].rs) | ((uint64_t)pack2_bf16(fr[k][2].rs, fr[k][3].rs) << 32);
          }
        }
      }
      // e_int is the error of the magnitude; e carries the sign of x: (e_int ^ s) - s with s = -1 for x < 0, else 0
      auto add_one = [&](const FastRound& f, uint32_t bits) {
        const float y = fast_value<FMT>(f.rs);
        if constexpr (POSITIVE) {
          cur.se_i += f.e_int;
        } else {
          const int32_t s = (int32_t)bits >> 31;
          cur.se_i += f.e_int ^ s;
          cur.neg_i += s;
        }
        cur.see_i += (long long)f.e_int * (long long)f.e_int;
        if constexpr (SumYInFp32<FMT>::value) cur.sy32 += y;
        else cur.sy += (double)y;
      };
      over_bins(
          p * kStatsPairElems, kStatsPairElems,
          [&]() {
#pragma unroll
            for (int k = 0; k < kRows; ++k)
#pragma unroll
              for (int j = 0; j < 4; ++j) add_one(fr[k][j], b[k][j]);
          },
          [&](int first, int last) {
#pragma unroll
            for (int k = 0; k < kRows; ++k)
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                const int e = k * 256 + 4 * lane + j;
                // outside the range: a zero code with a zero error adds exact zeros
                const bool in = e >= first && e < last;
                FastRound f = fr[k][j];
                f.rs = in ? f.rs : 0u;
                f.e_int = in ? f.e_int : 0;
                add_one(f, b[k][j]);
              }
          });
    };
    if constexpr (kSaturates<FMT>::value) {
      if (path == kSaturated || path == kPositiveSaturated) {
        int32_t e20[kRows][4];
#pragma unroll
        for (int k = 0; k < kRows; ++k)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t u = b[k][j] & 0x7FFFFFFFu;
            const uint32_t m24 = (u & 0x007FFFFFu) | 0x00800000u;
            const int32_t mag = (int32_t)(7u << (156u - (u >> 23))) - (int32_t)m24;   // (M - |x|) / ulp_t(x) 2^20 <= 0
            const int32_t sgn = (int32_t)b[k][j] >> 31;
            e20[k][j] = (mag ^ sgn) - sgn;                                            // e carries the sign of x
          }
        if (out != nullptr) {
          const uint64_t orow = (span_lo - i0) / 4 + (uint64_t)(p * (kStatsPairElems / 4) + lane);
#pragma unroll
          for (int k = 0; k < kRows; ++k) {
            const uint32_t signs = pack4_fp8<FMT>(b[k][0], b[k][1], b[k][2], b[k][3]) & 0x80808080u;
            reinterpret_cast<uint32_t*>(out)[orow + (uint64_t)(k * 64)] = signs | 0x7E7E7E7Eu;
          }
        }
        auto add_one = [&](int32_t e, uint32_t bits, bool in) {
          cur.se20_i += in ? e : 0;
          cur.see20_i += (long long)(in ? e : 0) * (long long)(in ? e : 0);
          const float y = __uint_as_float((bits & 0x80000000u) | F::U_MAXFIN);
          cur.sy32 += in ? y : 0.0f;
        };
        over_bins(
            p * kStatsPairElems, kStatsPairElems,
            [&]() {
#pragma unroll
              for (int k = 0; k < kRows; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) add_one(e20[k][j], b[k][j], true);
            },
            [&](int first, int last) {
#pragma unroll
              for (int k = 0; k < kRows; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                  const int e = k * 256 + 4 * lane + j;
                  add_one(e20[k][j], b[k][j], e >= first && e < last);
                }
            });
        return;
      }
    }
    typedef std::integral_constant<bool, F::kIsFp8> fp8_tag;
    if (path == kPositive) integer_pair(std::false_type{}, std::true_type{}, std::false_type{});
    else if (path == kSigned) integer_pair(std::false_type{}, std::false_type{}, std::false_type{});
    else if (path == kPositiveMixed) integer_pair(fp8_tag{}, std::true_type{}, std::false_type{});
    else if (path == kPositiveSubnormal) integer_pair(fp8_tag{}, std::true_type{}, fp8_tag{});
    else integer_pair(fp8_tag{}, std::false_type{}, std::false_type{});
  };

  if (my_pairs > 0) {
    load_pair(va, 0, true);
    draw(0);
    // Two pairs per trip, their loads in two register sets: the loads of a pair are in flight while the pair before
    // it is worked on, and no register is copied.  Every trip issues its loads whether or not the pair exists (past
    // the end a single word is read and dropped): with a load that may or may not have been issued the compiler
    // would have to wait for all of them at the point where the two cases meet.
    const int last = my_pairs - 1;
#pragma unroll 1
    for (int p = 0; p < kStatsSpanPairs; p += 2) {
      load_pair(vb, p + 1, p + 1 <= last);
      if (p % PPR == 0 && p / PPR + 1 < (kStatsSpanPairs + PPR - 1) / PPR) draw(p / PPR + 1);
      do_pair(va, p);
      if (p + 1 > last) break;   // uniform over the wave
      load_pair(va, p + 2, p + 2 <= last);
      if ((p + 1) % PPR == 0 && (p + 1) / PPR + 1 < (kStatsSpanPairs + PPR - 1) / PPR) draw((p + 1) / PPR + 1);
      do_pair(vb, p + 1);
      if (p + 2 > last) break;
    }
    close_bin();
  }
  __syncthreads();
  const int t = threadIdx.x;
  if (t < nbins_here * (int)kStatsRecordDoubles) {
    const int s = t / (int)kStatsRecordDoubles, k = t % (int)kStatsRecordDoubles;
    double v = part[0][s][k];
#pragma unroll
    for (int wv = 1; wv < kWavesPerBlock; ++wv) v += part[wv][s][k];
    if (s == 0) {
      records[chunk * (2 * kStatsRecordDoubles) + k] = v;
    } else if (s == nbins_here - 1) {
      records[chunk * (2 * kStatsRecordDoubles) + kStatsRecordDoubles + k] = v;
    } else {
      double* st = stats + (bin_first + (uint64_t)s - first_bin) * 4;   // a bin that lies inside this chunk: no other writer
      st[1 + k] += v;
      if (k == 0) st[0] += (double)group;
    }
  }
}

// One wave per bin: adds up the parts of the bin that stats_spans left in the workspace (the bin is the first or the
// last one of every chunk it shares with a neighbour; a bin inside a single chunk was finished there) and adds the
// totals to the caller's statistics.  Chunks cover global indices [i0, i_end).
__global__ __launch_bounds__(64) void stats_finalize(const double* __restrict__ records, uint64_t i0, uint64_t i_end,
                                                     uint64_t group, uint64_t bin_lo, uint64_t first_bin,
                                                     double* __restrict__ stats) {
  const int lane = threadIdx.x;
  const uint64_t bin = bin_lo + blockIdx.x;
  const uint64_t lo = bin * group > i0 ? bin * group : i0;
  const uint64_t be = bin_end(bin, group);
  const uint64_t hi = be < i_end ? be : i_end;
  if (lo >= hi) return;
  const uint64_t c_lo = (lo - i0) / kStatsChunkElems, c_hi = (hi - 1 - i0) / kStatsChunkElems;
  double sy = 0.0, se = 0.0, see = 0.0;
  bool mine = false;
  for (uint64_t c = c_lo + (uint64_t)lane; c <= c_hi; c += 64) {
    const uint64_t cs = i0 + c * kStatsChunkElems;
    const uint64_t ce = cs + kStatsChunkElems < i_end ? cs + kStatsChunkElems : i_end;
    const uint64_t fb = cs / group, lb = (ce - 1) / group;
    if (bin != fb && bin != lb) continue;   // inside chunk c (then c_lo == c_hi): finished by stats_spans
    const double* rec = records + c * (2 * kStatsRecordDoubles) + (bin == fb ? 0 : kStatsRecordDoubles);
    sy += rec[0];
    se += rec[1];
    see += rec[2];
    mine = true;
  }
  if (!__any(mine)) return;
  sy = wave_total(sy);
  se = wave_total(se);
  see = wave_total(see);
  if (lane == 0) {
    double* s = stats + (bin - first_bin) * 4;
    s[0] += (double)(hi - lo);
    s[1] += sy;
    s[2] += se;
    s[3] += see;
  }
}

// One thread per bin, serial over the bin's elements inside [a, a + n): any alignment, any
// group size; used for ragged heads and tails and for bins shorter than kStatsMinGroup.
template <int FMT, int VAR>
__global__ __launch_bounds__(kThreads) void stats_bins(const float* __restrict__ x, void* __restrict__ out, uint64_t n,
                                                       int nbits, int W, int log2_per_block, uint64_t seed, uint64_t a0,
                                                       uint64_t group, uint64_t bin_lo, uint64_t nb, uint64_t first_bin,
                                                       double* __restrict__ stats) {
  const uint64_t k = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k >= nb) return;
  const uint64_t bin = bin_lo + k;
  const uint64_t lo = bin * group > a0 ? bin * group : a0;
  const uint64_t be = bin_end(bin, group);
  const uint64_t hi = be < a0 + n ? be : a0 + n;
  if (lo >= hi) return;
  const bool many_bits = VAR != kRNE && nbits > kMaxTileNbits;   // uniform over the launch
  const Addends a = make_addends<FMT, VAR>(many_bits ? kMaxTileNbits : nbits);
  double sy = 0.0, se = 0.0, see = 0.0;
  typedef typename Fx<FMT>::code_t code_t;
  for (uint64_t i = lo; i < hi; ++i) {
    const uint32_t bits = __float_as_uint(x[i - a0]);
    uint32_t r;
    if constexpr (VAR != kRNE) {
      const uint32_t rnd = element_bits(i, log2_per_block, W, (uint32_t)nbits, seed, 0);
      r = many_bits ? round_pattern_wide<FMT, VAR>(bits, rnd, (uint32_t)nbits) : round_pattern<FMT, VAR, true>(bits, rnd, a);
    } else {
      r = round_pattern<FMT, VAR, true>(bits, 0u, a);
    }
    if (out != nullptr) reinterpret_cast<code_t*>(out)[i - a0] = (code_t)(r >> Fx<FMT>::FRAC);
    const double y = (double)decode_top<FMT>(r);
    const double e = (y - (double)__uint_as_float(bits)) * inv_ulp<FMT>(bits);
    sy += y;
    se += e;
    see = fma(e, e, see);
  }
  double* s = stats + (bin - first_bin) * 4;
  s[0] += (double)(hi - lo);
  s[1] += sy;
  s[2] += se;
  s[3] += see;
}

namespace {

template <int FMT, int VAR, int W>
hipError_t launch_spans(const float* x, void* out, uint64_t npairs, int nbits, uint64_t seed, uint64_t blk0,
                        uint64_t i0, uint64_t group, uint64_t first_bin, double* records, double* stats,
                        hipStream_t stream) {
  const uint64_t per_chunk = kStatsChunkElems / kStatsPairElems;
  const uint64_t chunks = (npairs + per_chunk - 1) / per_chunk;
  for (uint64_t c0 = 0; c0 < chunks; c0 += kMaxTilesPerLaunch) {   // at most 2^30 threads per launch
    const uint64_t cnt = chunks - c0 < kMaxTilesPerLaunch ? chunks - c0 : kMaxTilesPerLaunch;
    hipLaunchKernelGGL((stats_spans<FMT, VAR, W>), dim3((unsigned)cnt), dim3(kThreads), 0, stream, x, out, npairs, nbits,
                       seed, blk0, i0, group, first_bin, c0, records, stats);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int FMT, int VAR>
hipError_t launch_spans_w(int W, const float* x, void* out, uint64_t npairs, int nbits, uint64_t seed, uint64_t blk0,
                          uint64_t i0, uint64_t group, uint64_t first_bin, double* records, double* stats,
                          hipStream_t stream) {
  if constexpr (VAR == kRNE) {
    return launch_spans<FMT, VAR, 8>(x, out, npairs, nbits, seed, blk0, i0, group, first_bin, records, stats, stream);
  } else {
    switch (W) {
      case 1: return launch_spans<FMT, VAR, 1>(x, out, npairs, nbits, seed, blk0, i0, group, first_bin, records, stats, stream);
      case 2: return launch_spans<FMT, VAR, 2>(x, out, npairs, nbits, seed, blk0, i0, group, first_bin, records, stats, stream);
      case 4: return launch_spans<FMT, VAR, 4>(x, out, npairs, nbits, seed, blk0, i0, group, first_bin, records, stats, stream);
      case 8: return launch_spans<FMT, VAR, 8>(x, out, npairs, nbits, seed, blk0, i0, group, first_bin, records, stats, stream);
      case 16: return launch_spans<FMT, VAR, 16>(x, out, npairs, nbits, seed, blk0, i0, group, first_bin, records, stats, stream);
      default: return launch_spans<FMT, VAR, 32>(x, out, npairs, nbits, seed, blk0, i0, group, first_bin, records, stats, stream);
    }
  }
}

// Per-bin kernel over the n elements whose first global index is a0.
template <int FMT, int VAR>
hipError_t launch_bins(const float* x, void* out, uint64_t n, int nbits, int W, uint64_t seed, uint64_t a0,
                       uint64_t group, uint64_t first_bin, double* stats, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint64_t bin_lo = a0 / group, bin_hi = (a0 + n - 1) / group;
  const uint64_t nb = bin_hi - bin_lo + 1;
  for (uint64_t at = 0; at < nb; at += kMaxElemsPerLaunch) {
    const uint64_t m = nb - at < kMaxElemsPerLaunch ? nb - at : kMaxElemsPerLaunch;
    const uint64_t blocks = (m + kThreads - 1) / kThreads;
    hipLaunchKernelGGL((stats_bins<FMT, VAR>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, x, out, n, nbits, W,
                       log2_of(128 / W), seed, a0, group, bin_lo + at, m, first_bin, stats);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int FMT, int VAR>
hipError_t run(const float* x, void* out, uint64_t n, int nbits, uint64_t seed, uint64_t offset, uint64_t group,
               uint64_t first_bin, double* stats, double* workspace, hipStream_t stream) {
  const int W = VAR == kRNE ? 8 : slot_width(nbits);
  const uint64_t osize = sizeof(typename Fx<FMT>::code_t);
  // the vector kernel takes whole pairs of rows, from the first element that starts a Philox block
  const Split s = split_range(n, offset, W, VAR == kRNE, reinterpret_cast<uintptr_t>(x), 4, 16,
                              reinterpret_cast<uintptr_t>(out), osize, 4 * osize, 0, 0, 1, kStatsPairElems);
  const uint64_t head = group < kStatsMinGroup ? 0 : s.head;
  const uint64_t npairs = group < kStatsMinGroup ? 0 : s.ntiles;
  char* o = reinterpret_cast<char*>(out);
  hipError_t e = launch_bins<FMT, VAR>(x, out, head, nbits, W, seed, offset, group, first_bin, stats, stream);
  if (e != hipSuccess) return e;
  if (npairs) {
    const uint64_t i0 = offset + head;
    e = launch_spans_w<FMT, VAR>(W, x + head, out ? o + head * osize : nullptr, npairs, nbits, seed,
                                 i0 / (uint64_t)(128 / W), i0, group, first_bin, workspace, stats, stream);
    if (e != hipSuccess) return e;
    e = launch_stats_finalize(workspace, i0, i0 + npairs * kStatsPairElems, group, first_bin, stats, stream);
    if (e != hipSuccess) return e;
  }
  const uint64_t done = head + npairs * kStatsPairElems;
  return launch_bins<FMT, VAR>(x + done, out ? o + done * osize : nullptr, n - done, nbits, W, seed, offset + done,
                               group, first_bin, stats, stream);
}

template <int FMT>
hipError_t run_v(int variant, const float* x, void* out, uint64_t n, int nbits, uint64_t seed, uint64_t offset,
                 uint64_t group, uint64_t first_bin, double* stats, double* workspace, hipStream_t stream) {
  switch (variant) {
    case kRNE: return run<FMT, kRNE>(x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
    case kSRFF: return run<FMT, kSRFF>(x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
    case kSRF: return run<FMT, kSRF>(x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
    default: return run<FMT, kSRC>(x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
  }
}

}  // namespace

hipError_t launch_stats_finalize(const double* records, uint64_t i0, uint64_t i_end, uint64_t group, uint64_t first_bin,
                                 double* stats, hipStream_t stream) {
  const uint64_t bin_lo = i0 / group, bin_hi = (i_end - 1) / group;
  for (uint64_t at = 0; at <= bin_hi - bin_lo; at += kMaxElemsPerLaunch) {
    const uint64_t m = bin_hi - bin_lo + 1 - at < kMaxElemsPerLaunch ? bin_hi - bin_lo + 1 - at : kMaxElemsPerLaunch;
    hipLaunchKernelGGL(stats_finalize, dim3((unsigned)m), dim3(64), 0, stream, records, i0, i_end, group, bin_lo + at, first_bin,
                       stats);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Workspace for callers that cannot allocate one: a fixed array in the library's device image.  Every GPU the
// library runs on holds its own copy at its own address for the life of the process.  In host code the array's
// name is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_lock;
void* scratch_of_device[kMaxDevices];   // the array's address on each device, looked up on that device's first call
}  // namespace

hipError_t static_scratch(double** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(scratch_lock);
  if (scratch_of_device[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // of the current device
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    scratch_of_device[dev] = p;
  }
  *ptr = reinterpret_cast<double*>(scratch_of_device[dev]);
  return hipSuccess;
}

hipError_t launch_stats(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
                        uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins, double* stats,
                        double* workspace, hipStream_t stream) {
  (void)nbins;
  switch (fmt) {
    case kBF16: return run_v<kBF16>(variant, x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
    case kE4M3: return run_v<kE4M3>(variant, x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
    case kE5M2: return run_v<kE5M2>(variant, x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
    default: return run_v<kP4>(variant, x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
  }
}

}  // namespace fbsr
