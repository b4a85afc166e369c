// fbsr_stats.hip -- kernels behind fbsr_bias_stats: round as fbsr_round and reduce, per bin,
// {count, sum y, sum e, sum e^2} with y the decoded rounded value and e = (y - x) / ulp_t(x)
// in fp64 -- the measurement behind Figs. 1 and 2 (mean rounded value per input, bias in
// target ulps, Sec. III).  Bins are runs of `group` consecutive global indices.
//
// Reduction order is fixed (lane-local sums -> xor-butterfly across the wave -> the four waves'
// sums staged in LDS and added in wave order -> one record per (chunk, bin) in the workspace ->
// per-bin sums over its chunks, lane-strided then butterfly), so results are bit-reproducible;
// no floating-point atomics are used.
#include <mutex>
#include <type_traits>

#include "fbsr_launch.h"

namespace fbsr {

struct Acc {
  double sy, se, see;   // sum y, sum e, sum e^2
  float sy32;           // the part of sum y kept in fp32 (formats whose sums over a chunk are exact there)
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Decoded value of the signed code held in the top bits of r (Eq. (1)).
template <int FMT>
__device__ __forceinline__ float decode_top(uint32_t r) {
  typedef Fx<FMT> F;
  if constexpr (!F::kIsFp8) {
    return __uint_as_float(r & 0xFFFF0000u);
  } else if constexpr (FMT == kP4) {
    return fp8_code_value<kP4>(r >> 24);
  } else {
    const uint32_t c = (r >> 24) & 0x7Fu;
    const uint32_t e = c >> (F::P - 1);
    const uint32_t t = c & ((1u << (F::P - 1)) - 1u);
    const uint32_t mant = e ? (t | (1u << (F::P - 1))) : t;       // subnormals have no hidden one
    const int ex = (int)(e ? e : 1u) - (F::B + F::P - 1);
    float y = ldexpf((float)mant, ex);
    if constexpr (FMT == kE5M2) {
      y = c == F::INF_CODE ? __uint_as_float(0x7F800000u) : y;
      y = c > F::INF_CODE ? __uint_as_float(0x7FC00000u) : y;
    } else {
      y = c == 0x7Fu ? __uint_as_float(0x7FC00000u) : y;
    }
    return __uint_as_float(__float_as_uint(y) | (r & 0x80000000u));
  }
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

// A lane's share of a chunk is 64 elements.  64 values of E4M3 (multiples of 2^-9 up to 448) or of binary8p4
// (multiples of 2^-10 up to 224) sum to a multiple of that step below 2^24 steps: exact in fp32 in any order, so
// the sum of y runs there and is widened once per record.
template <int FMT> struct SumYInFp32 { static constexpr bool value = FMT == kE4M3 || FMT == kP4; };

// Adds one element to a bin's sums.  WIDE = false: y - x is formed in fp32, where it is exact for
// every finite |x| <= M (y is a neighbour of x on a coarser grid, so the difference is a multiple of
// x's own last place and smaller than 2^24 of them), and so is its scaling by 1 / ulp_t(x), a power of two
// (the quotient keeps the difference's significand and stays below 2 in magnitude);
// WIDE = true: the difference is formed in fp64 (overflow, saturation, NaN: values for which the fp32 difference
// would round or is not finite).  Either way e = (y - x) / ulp_t(x) reaches the fp64 sums without a rounding.
template <int FMT, bool WIDE>
__device__ __forceinline__ void accumulate(Acc& acc, uint32_t bits, float y) {
  typedef Fx<FMT> F;
  const float x = __uint_as_float(bits);
  double e;
  if constexpr (WIDE) {
    e = ((double)y - (double)x) * inv_ulp<FMT>(bits);
    acc.sy += (double)y;
  } else {
    // 1 / ulp_t(x) = 2^(P - 1 - e~), e~ = max(floor(log2|x|), 1 - B) (Eq. (2)); frexp's exponent is floor(log2|x|) + 1
    // (0 for x = 0, where y - x = 0 makes the scale irrelevant)
    const int fe = __builtin_amdgcn_frexp_expf(x);
    const int k = F::P - (fe > 2 - F::B ? fe : 2 - F::B);
    e = (double)__builtin_amdgcn_ldexpf(y - x, k);
    if constexpr (SumYInFp32<FMT>::value) acc.sy32 += y;
    else acc.sy += (double)y;
  }
  acc.se += e;
  acc.see = fma(e, e, acc.see);
}

// The four decoded values of a packed fp8 word (the hardware decode equals Eq. (1) on all 256 codes).
template <int FMT>
__device__ __forceinline__ void decode4(uint32_t packed, float (&y)[4]) {
  if constexpr (FMT == kE4M3 || FMT == kP4) {
    y[0] = __builtin_amdgcn_cvt_f32_fp8((int)packed, 0); y[1] = __builtin_amdgcn_cvt_f32_fp8((int)packed, 1);
    y[2] = __builtin_amdgcn_cvt_f32_fp8((int)packed, 2); y[3] = __builtin_amdgcn_cvt_f32_fp8((int)packed, 3);
    if constexpr (FMT == kP4) {   // finite binary8p4 values are one half of E4M3's at the same code
#pragma unroll
      for (int j = 0; j < 4; ++j) y[j] *= 0.5f;
    }
  } else {
    y[0] = __builtin_amdgcn_cvt_f32_bf8((int)packed, 0); y[1] = __builtin_amdgcn_cvt_f32_bf8((int)packed, 1);
    y[2] = __builtin_amdgcn_cvt_f32_bf8((int)packed, 2); y[3] = __builtin_amdgcn_cvt_f32_bf8((int)packed, 3);
  }
}

// One workgroup per chunk of kStatsChunkTiles tiles.  Sums run in registers across the chunk's
// tiles and are flushed (wave butterfly -> LDS -> record) when a bin ends and at the chunk's end:
// record (chunk c, slot s) holds the chunk's part of bin floor(start(c) / group) + s.
// The random bits of the whole chunk are drawn first, its Philox blocks dealt round-robin to all 256
// threads (a tile alone has work for 16 W of them, which would leave most waves waiting), and one barrier
// publishes them; after that the four waves walk the chunk's tiles independently.
template <int FMT, int VAR, int W>
__global__ __launch_bounds__(kThreads) void stats_tiles(const float* __restrict__ x, void* __restrict__ out,
                                                        uint64_t ntiles, int nbits, uint64_t seed, uint64_t blk0,
                                                        uint64_t i0, uint64_t group, uint64_t slots,
                                                        double* __restrict__ records) {
  typedef WgTile<W> T;
  typedef Fx<FMT> F;
  // MANY: more than 16 random bits per element (32-bit slots, the wide rounding).  The strip then holds the bits of
  // half a chunk at a time (32 KiB) and is refilled before the fifth tile.
  constexpr bool MANY = W == 32 && VAR != kRNE;
  constexpr int kStripTiles = MANY ? kStatsChunkTiles / 2 : kStatsChunkTiles;
  __shared__ uint4 strip[kStripTiles * T::BLOCKS];
  __shared__ double staged[kWavesPerBlock][kStatsRecordDoubles];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;

  const Addends a = make_addends<FMT, VAR>(MANY ? kMaxTileNbits : nbits);
  HwAddends hw = {0, 0, 0, 0};
  if constexpr (F::kIsFp8 && VAR != kRNE && !MANY) hw = make_hw_addends<FMT, VAR>(nbits);
  const uint64_t tile0 = (uint64_t)blockIdx.x * kStatsChunkTiles;
  const uint64_t chunk_start = i0 + tile0 * T::ELEMS;
  uint64_t next_bin = group - chunk_start % group;   // chunk-relative index at which the next bin starts
  uint64_t slot = 0;
  Acc cur = {0.0, 0.0, 0.0, 0.0f};
  // draws the bits of the tiles [first, first + kStripTiles) of the chunk (those that exist) into the strip
  auto draw = [&](int first) {
    const uint64_t left = ntiles - (tile0 + (uint64_t)first);   // > 0 at every call
    const int nblk = (int)(left < (uint64_t)kStripTiles ? left : (uint64_t)kStripTiles) * T::BLOCKS;
    for (int bi = threadIdx.x; bi < nblk; bi += kThreads) {
      uint32_t o[4];
      philox_block(blk0 + (tile0 + (uint64_t)first) * T::BLOCKS + (uint64_t)bi, seed, 0, o);
      strip[bi] = make_uint4(o[0], o[1], o[2], o[3]);
    }
    __syncthreads();
  };
  if constexpr (VAR != kRNE) draw(0);   // the grid has one workgroup per started chunk: tile0 < ntiles

  auto flush = [&]() {
    const double t0 = wave_sum(cur.sy + (double)cur.sy32), t1 = wave_sum(cur.se), t2 = wave_sum(cur.see);
    if (lane == 0) {
      staged[wave][0] = t0; staged[wave][1] = t1; staged[wave][2] = t2;
    }
    __syncthreads();
    if (threadIdx.x < kStatsRecordDoubles) {
      double t = staged[0][threadIdx.x];
#pragma unroll
      for (int wv = 1; wv < kWavesPerBlock; ++wv) t += staged[wv][threadIdx.x];
      records[((uint64_t)blockIdx.x * slots + slot) * kStatsRecordDoubles + threadIdx.x] = t;
    }
    __syncthreads();
    slot += 1;
    cur = {0.0, 0.0, 0.0, 0.0f};
  };

  // the loads of a tile are issued one iteration ahead, so that their latency is covered by the arithmetic of
  // the tile before (the waves of a workgroup run independently between the chunk's barriers)
  const uint64_t lane_row = (uint64_t)(wave * (kWaveElems / 4) + lane);
  f32x4 ahead[kRows];
#pragma unroll
  for (int k = 0; k < kRows; ++k) ahead[k] = load_stream4(x + 4 * (tile0 * (T::ELEMS / 4) + lane_row + (uint64_t)(k * 64)));   // tile0 < ntiles
#pragma unroll 1
  for (int it = 0; it < kStatsChunkTiles; ++it) {
    const uint64_t tile = tile0 + (uint64_t)it;
    if (tile >= ntiles) break;   // uniform over the workgroup
    if constexpr (MANY) {
      if (it == kStripTiles) {   // every wave is done with the first half's bits before they are replaced
        __syncthreads();
        draw(kStripTiles);
      }
    }
    const uint64_t row0 = tile * (T::ELEMS / 4) + lane_row;   // units of 4 elements
    f32x4 v[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) v[k] = ahead[k];
    if (it + 1 < kStatsChunkTiles && tile + 1 < ntiles) {
#pragma unroll
      for (int k = 0; k < kRows; ++k) ahead[k] = load_stream4(x + 4 * (row0 + (uint64_t)(T::ELEMS / 4) + (uint64_t)(k * 64)));
    }

    uint32_t b[kRows][4];
    float y[kRows][4];
    uint32_t umax = 0;
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
      b[k][0] = __float_as_uint(v[k].x); b[k][1] = __float_as_uint(v[k].y);
      b[k][2] = __float_as_uint(v[k].z); b[k][3] = __float_as_uint(v[k].w);
#pragma unroll
      for (int j = 0; j < 4; ++j) umax = max(umax, b[k][j] & 0x7FFFFFFFu);
    }
    // wave-uniform: |x| > M or NaN anywhere in the wave sends it down the checked integer rounding and
    // the fp64 difference; otherwise the unchecked rounding (hardware converts for fp8) applies
    const bool wide_path = __any(umax > F::U_MAXFIN);
    const uint64_t t_lo = (uint64_t)it * T::ELEMS, t_hi = t_lo + T::ELEMS;   // chunk-relative range of this tile

    // the rest of the tile, instantiated once per flavour so that each is straight-line code
    auto finish_tile = [&](auto wide_tag) {
      constexpr bool WIDE = decltype(wide_tag)::value;
#pragma unroll
      for (int k = 0; k < kRows; ++k) {
        uint32_t n4[4] = {0, 0, 0, 0};
        if constexpr (MANY) {
          // the row's four 32-bit slots are one Philox block
          const uint4 q = strip[(it % kStripTiles) * T::BLOCKS + (wave * kWaveElems + k * 256 + 4 * lane) / 4];
          n4[0] = __builtin_amdgcn_ubfe(q.x, 0u, (uint32_t)nbits); n4[1] = __builtin_amdgcn_ubfe(q.y, 0u, (uint32_t)nbits);
          n4[2] = __builtin_amdgcn_ubfe(q.z, 0u, (uint32_t)nbits); n4[3] = __builtin_amdgcn_ubfe(q.w, 0u, (uint32_t)nbits);
        } else if constexpr (VAR != kRNE) {
          const uint64_t rb = read_wg_row_bits<W>(strip + it * T::BLOCKS, wave, lane, k);
#pragma unroll
          for (int j = 0; j < 4; ++j) n4[j] = slot_bits<W>(rb, j, a.nbits);
        }
        constexpr bool HW = !WIDE && F::kIsFp8 && VAR != kRNE && !MANY;
        uint32_t r[4] = {0, 0, 0, 0};
        uint32_t packed = 0;
        if constexpr (HW) {
          packed = round4_fp8_hw<FMT, VAR>(b[k], n4, hw);
        } else if constexpr (MANY) {
#pragma unroll
          for (int j = 0; j < 4; ++j) r[j] = round_pattern_wide<FMT, VAR>(b[k][j], n4[j], (uint32_t)nbits);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) r[j] = round_pattern<FMT, VAR, WIDE>(b[k][j], n4[j], a);
        }
        const uint64_t row = row0 + (uint64_t)(k * 64);
        if constexpr (F::kIsFp8) {
          if constexpr (!HW) packed = pack4_fp8<FMT>(r[0], r[1], r[2], r[3]);
          if constexpr (WIDE) {
#pragma unroll
            for (int j = 0; j < 4; ++j) y[k][j] = decode_top<FMT>(r[j]);   // keeps this library's NaN / sign conventions
          } else {
            decode4<FMT>(packed, y[k]);
          }
          if (out != nullptr) reinterpret_cast<uint32_t*>(out)[row] = packed;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) y[k][j] = __uint_as_float(r[j] & 0xFFFF0000u);
          if (out != nullptr)
            reinterpret_cast<uint64_t*>(out)[row] = (uint64_t)pack2_bf16(r[0], r[1]) | ((uint64_t)pack2_bf16(r[2], r[3]) << 32);
        }
      }

      // adds the elements whose tile-relative index lies in [lo, hi) to `cur`; ALL = the whole tile
      auto add_range = [&](auto all_tag, int lo, int hi) {
        constexpr bool ALL = decltype(all_tag)::value;
        const int w_lo = wave * kWaveElems;
#pragma unroll
        for (int k = 0; k < kRows; ++k)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int e = w_lo + k * 256 + 4 * lane + j;
            const bool in = ALL || (e >= lo && e < hi);
            if constexpr (ALL) {
              accumulate<FMT, WIDE>(cur, b[k][j], y[k][j]);
            } else if constexpr (WIDE) {
              if (in) accumulate<FMT, true>(cur, b[k][j], y[k][j]);
            } else {
              // outside the range: contribute y = 0 and x = 0, whose terms are exact zeros
              accumulate<FMT, false>(cur, in ? b[k][j] : 0u, in ? y[k][j] : 0.0f);
            }
          }
      };

      if (next_bin >= t_hi) {
        add_range(std::true_type{}, 0, T::ELEMS);
      } else {                       // a bin ends inside this tile (at most once: group >= tile)
        const int cut = (int)(next_bin - t_lo);
        add_range(std::false_type{}, 0, cut);
        flush();
        add_range(std::false_type{}, cut, T::ELEMS);
        next_bin += group;
      }
    };
    if (wide_path) finish_tile(std::true_type{});
    else finish_tile(std::false_type{});
  }
  flush();
}

// One wave per bin: sums the records of the chunks that overlap the bin and adds the bin's totals
// to the caller's statistics.  Chunks cover global indices [i0, i_end).
__global__ __launch_bounds__(64) void stats_finalize(const double* __restrict__ records, uint64_t i0, uint64_t i_end,
                                                     uint64_t chunk_elems, uint64_t slots, uint64_t group,
                                                     uint64_t bin_lo, uint64_t first_bin, double* __restrict__ stats) {
  const int lane = threadIdx.x;
  const uint64_t bin = bin_lo + blockIdx.x;
  const uint64_t lo = bin * group > i0 ? bin * group : i0;
  const uint64_t hi = (bin + 1) * group < i_end ? (bin + 1) * group : i_end;
  if (lo >= hi) return;
  const uint64_t c_lo = (lo - i0) / chunk_elems, c_hi = (hi - 1 - i0) / chunk_elems;
  double sy = 0.0, se = 0.0, see = 0.0;
  for (uint64_t c = c_lo + (uint64_t)lane; c <= c_hi; c += 64) {
    const uint64_t first = (i0 + c * chunk_elems) / group;   // the bin of the chunk's slot 0
    const double* rec = records + (c * slots + (bin - first)) * kStatsRecordDoubles;
    sy += rec[0];
    se += rec[1];
    see += rec[2];
  }
  sy = wave_sum(sy);
  se = wave_sum(se);
  see = wave_sum(see);
  if (lane == 0) {
    double* s = stats + (bin - first_bin) * 4;
    s[0] += (double)(hi - lo);
    s[1] += sy;
    s[2] += se;
    s[3] += see;
  }
}

// One thread per bin, serial over the bin's elements inside [a, a + n): any alignment, any
// group size; used for ragged heads and tails and whenever the tile kernel does not apply.
template <int FMT, int VAR>
__global__ __launch_bounds__(kThreads) void stats_bins(const float* __restrict__ x, void* __restrict__ out, uint64_t n,
                                                       int nbits, int W, int log2_per_block, uint64_t seed, uint64_t a0,
                                                       uint64_t group, uint64_t bin_lo, uint64_t nb, uint64_t first_bin,
                                                       double* __restrict__ stats) {
  const uint64_t k = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k >= nb) return;
  const uint64_t bin = bin_lo + k;
  const uint64_t lo = bin * group > a0 ? bin * group : a0;
  const uint64_t hi = (bin + 1) * group < a0 + n ? (bin + 1) * group : a0 + n;
  if (lo >= hi) return;
  const bool many_bits = VAR != kRNE && nbits > kMaxTileNbits;   // uniform over the launch
  const Addends a = make_addends<FMT, VAR>(many_bits ? kMaxTileNbits : nbits);
  Acc acc = {0.0, 0.0, 0.0, 0.0f};
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
    accumulate<FMT, true>(acc, bits, decode_top<FMT>(r));
  }
  double* s = stats + (bin - first_bin) * 4;
  s[0] += (double)(hi - lo);
  s[1] += acc.sy;
  s[2] += acc.se;
  s[3] += acc.see;
}

namespace {

template <int FMT, int VAR, int W>
hipError_t launch_tiles(const float* x, void* out, uint64_t ntiles, int nbits, uint64_t seed, uint64_t blk0,
                        uint64_t i0, uint64_t group, double* records, hipStream_t stream) {
  const uint64_t chunks = (ntiles + kStatsChunkTiles - 1) / kStatsChunkTiles;
  const uint64_t slots = stats_slots(group);
  const uint64_t osize = sizeof(typename Fx<FMT>::code_t);
  for (uint64_t c0 = 0; c0 < chunks; c0 += kMaxTilesPerLaunch) {   // at most 2^30 threads per launch
    const uint64_t cnt = chunks - c0 < kMaxTilesPerLaunch ? chunks - c0 : kMaxTilesPerLaunch;
    const uint64_t t0 = c0 * kStatsChunkTiles, e0 = t0 * kTileElems;
    hipLaunchKernelGGL((stats_tiles<FMT, VAR, W>), dim3((unsigned)cnt), dim3(kThreads), 0, stream, x + e0,
                       out ? reinterpret_cast<char*>(out) + e0 * osize : nullptr, ntiles - t0, nbits, seed,
                       blk0 + t0 * WgTile<W>::BLOCKS, i0 + e0, group, slots, records + c0 * slots * kStatsRecordDoubles);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int FMT, int VAR>
hipError_t launch_tiles_w(int W, const float* x, void* out, uint64_t ntiles, int nbits, uint64_t seed,
                          uint64_t blk0, uint64_t i0, uint64_t group, double* records, hipStream_t stream) {
  if constexpr (VAR == kRNE) {
    return launch_tiles<FMT, VAR, 8>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
  } else {
    switch (W) {
      case 1: return launch_tiles<FMT, VAR, 1>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
      case 2: return launch_tiles<FMT, VAR, 2>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
      case 4: return launch_tiles<FMT, VAR, 4>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
      case 8: return launch_tiles<FMT, VAR, 8>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
      case 16: return launch_tiles<FMT, VAR, 16>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
      default: return launch_tiles<FMT, VAR, 32>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
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
  Split s = split_range(n, offset, W, VAR == kRNE, reinterpret_cast<uintptr_t>(x), 4, 16,
                        reinterpret_cast<uintptr_t>(out), osize, 4 * osize);
  if (group < s.tile_elems) {   // a tile could touch more than two bins
    s.head = 0;
    s.ntiles = 0;
  }
  char* o = reinterpret_cast<char*>(out);
  hipError_t e = launch_bins<FMT, VAR>(x, out, s.head, nbits, W, seed, offset, group, first_bin, stats, stream);
  if (e != hipSuccess) return e;
  if (s.ntiles) {
    const uint64_t i0 = offset + s.head;
    e = launch_tiles_w<FMT, VAR>(W, x + s.head, out ? o + s.head * osize : nullptr, s.ntiles, nbits, seed,
                                 i0 / (uint64_t)(128 / W), i0, group, workspace, stream);
    if (e != hipSuccess) return e;
    const uint64_t bin_lo = i0 / group, bin_hi = (i0 + s.ntiles * s.tile_elems - 1) / group;
    hipLaunchKernelGGL(stats_finalize, dim3((unsigned)(bin_hi - bin_lo + 1)), dim3(64), 0, stream, workspace, i0,
                       i0 + s.ntiles * s.tile_elems, (uint64_t)kStatsChunkTiles * s.tile_elems, stats_slots(group), group,
                       bin_lo, first_bin, stats);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const uint64_t done = s.head + s.ntiles * s.tile_elems;
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
