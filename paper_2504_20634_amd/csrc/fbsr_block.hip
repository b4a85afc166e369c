// fbsr_block.hip -- kernels behind fbsr_round_block_scaled: fp32 -> fp8 with one power-of-two scale
// per block of 32 elements (the scaled-tensor layout of Sec. I-A), each element rounded by few-bit
// stochastic rounding after the exact scaling.
#include "fbsr_launch.h"

namespace fbsr {

constexpr int kScaleBlock = 32;

template <int FMT> struct Emax;
template <> struct Emax<kE4M3> { static constexpr int value = 8; };
template <> struct Emax<kE5M2> { static constexpr int value = 15; };
template <> struct Emax<kP4> { static constexpr int value = 7; };

// From the largest |x| pattern of a block: the scale exponent s (clamped to [-127, 127]) and whether
// the block holds a NaN or an infinity.  A pattern's exponent field is floor(log2) + 127 for normal
// values; fields of 0 (zero, fp32 subnormals) fall below the clamp whatever their exact logarithm.
template <int FMT>
__device__ __forceinline__ int scale_exponent(uint32_t umax, bool* special) {
  *special = umax >= 0x7F800000u;
  const int s = (int)(umax >> 23) - 127 - Emax<FMT>::value;
  return s < -127 ? -127 : s;   // the upper clamp cannot bind: fields stop at 254
}

// 2^-s as an fp32 value (s in [-127, 119]: always a normal number).
__device__ __forceinline__ float inv_scale(int s) { return __uint_as_float((uint32_t)(127 - s) << 23); }

// Same workgroup tile as fbsr_round (2048 elements, 2 rows of 4 elements per lane).  A block of 32
// elements is 8 adjacent lanes of one row: their maxima are combined with three xor-shuffles.
template <int FMT, int VAR, int W>
__global__ __launch_bounds__(kThreads) void block_tiles(const float* __restrict__ x, uint8_t* __restrict__ out,
                                                        uint8_t* __restrict__ scales, int nbits, uint64_t seed,
                                                        uint64_t blk0, uint32_t xcd_lg) {
  typedef WgTile<W> T;
  typedef Fx<FMT> F;
  __shared__ uint4 strip[T::BLOCKS];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x, xcd_lg);
  const uint64_t row0 = (uint64_t)tile * (T::ELEMS / 4) + (uint64_t)(wave * (kWaveElems / 4) + lane);   // units of 4 elements
  f32x4 v[kRows];
#pragma unroll
  for (int k = 0; k < kRows; ++k) v[k] = load_stream4(x + 4 * (row0 + (uint64_t)(k * 64)));
  if constexpr (VAR != kRNE) {
    fill_wg_bits<W>(strip, threadIdx.x, blk0 + (uint64_t)tile * T::BLOCKS, seed, 0);
    __syncthreads();
  }
  constexpr bool MANY = W == 32;   // more than 16 random bits: 32-bit slots
  const Addends a = make_addends<FMT, VAR>(MANY ? kMaxTileNbits : nbits);
  ManyAddends many = {a, 0.0f};
  if constexpr (MANY && VAR != kRNE) many = make_many_addends<FMT, VAR>(nbits);
  HwAddends hw = {0, 0, 0, 0};
  if constexpr (VAR != kRNE) hw = make_hw_addends<FMT, VAR>(nbits);
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    const uint32_t raw[4] = {__float_as_uint(v[k].x), __float_as_uint(v[k].y), __float_as_uint(v[k].z),
                             __float_as_uint(v[k].w)};
    uint32_t umax = max(max(raw[0] & 0x7FFFFFFFu, raw[1] & 0x7FFFFFFFu), max(raw[2] & 0x7FFFFFFFu, raw[3] & 0x7FFFFFFFu));
    // maximum over the 8 lanes of the block, by data-parallel-primitive moves (no LDS): neighbours within a quad,
    // the other pair of the quad, then the mirror image within the group of 8 (lane i <-> 7 - i: the other quad)
    umax = max(umax, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)umax, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    umax = max(umax, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)umax, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    umax = max(umax, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)umax, 0x141, 0xF, 0xF, false));   // row_half_mirror
    bool special;
    const int s = scale_exponent<FMT>(umax, &special);
    const float mult = inv_scale(s);
    uint32_t b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = special ? 0u : __float_as_uint(__uint_as_float(raw[j]) * mult);
    uint32_t packed;
    if constexpr (VAR != kRNE) {   // no NaN can reach the rounding: the hardware converts apply ...
      uint32_t n4[4];
      row_draws4<W>(strip, wave, lane, k, (uint32_t)nbits, n4);
      bool hw_ok = true;           // ... unless there are more random bits than they take on a value below the normal range
      if constexpr (MANY) {
        if (hw_needs_normal_inputs<FMT, VAR>(nbits)) {
          const uint32_t lowest = min(min(magnitude_less_one(b[0]), magnitude_less_one(b[1])),
                                      min(magnitude_less_one(b[2]), magnitude_less_one(b[3])));
          hw_ok = !__any(lowest < F::U_SUB - 1u);
        }
      }
      if (hw_ok) {
        packed = round4_fp8_hw<FMT, VAR, MANY>(b, n4, hw);
      } else {
        uint32_t r[4] = {0, 0, 0, 0};
        if constexpr (MANY) {
#pragma unroll
          for (int j = 0; j < 4; ++j) r[j] = round_pattern_many<FMT, VAR, false>(b[j], n4[j], (uint32_t)nbits, many);
        }
        packed = pack4_fp8<FMT>(r[0], r[1], r[2], r[3]);
      }
    } else {
      uint32_t r[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) r[j] = round_pattern<FMT, VAR, false>(b[j], 0u, a);
      packed = pack4_fp8<FMT>(r[0], r[1], r[2], r[3]);
    }
    constexpr uint32_t kNan4 = (F::NAN_FX >> 24) * 0x01010101u;
    packed = special ? kNan4 : packed;
    const uint64_t row = row0 + (uint64_t)(k * 64);
    __builtin_nontemporal_store(packed, reinterpret_cast<uint32_t*>(out) + row);
    if ((lane & 7) == 0) scales[row / (kScaleBlock / 4)] = special ? (uint8_t)0xFF : (uint8_t)(s + 127);
  }
}

// One thread per block of 32 (the last one may be short): any alignment, any offset, ragged tails.
template <int FMT, int VAR>
__global__ __launch_bounds__(kThreads) void block_blocks(const float* __restrict__ x, uint8_t* __restrict__ out,
                                                         uint8_t* __restrict__ scales, uint64_t n, int nbits, int W,
                                                         int log2_per_block, uint64_t seed, uint64_t offset) {
  const uint64_t blk = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  const uint64_t j0 = blk * kScaleBlock;
  if (j0 >= n) return;
  const int len = n - j0 < (uint64_t)kScaleBlock ? (int)(n - j0) : kScaleBlock;
  uint32_t umax = 0;
  for (int k = 0; k < len; ++k) umax = max(umax, __float_as_uint(x[j0 + k]) & 0x7FFFFFFFu);
  bool special;
  const int s = scale_exponent<FMT>(umax, &special);
  scales[blk] = special ? (uint8_t)0xFF : (uint8_t)(s + 127);
  const float mult = inv_scale(s);
  const bool many_bits = VAR != kRNE && nbits > kMaxTileNbits;   // uniform over the launch
  const Addends a = make_addends<FMT, VAR>(many_bits ? kMaxTileNbits : nbits);
  for (int k = 0; k < len; ++k) {
    const uint32_t bits = __float_as_uint(x[j0 + k] * mult);
    uint32_t r;
    if constexpr (VAR != kRNE) {
      const uint32_t rnd = element_bits(offset + j0 + k, log2_per_block, W, (uint32_t)nbits, seed, 0);
      r = many_bits ? round_pattern_wide<FMT, VAR>(bits, rnd, (uint32_t)nbits) : round_pattern<FMT, VAR, true>(bits, rnd, a);
    } else {
      r = round_pattern<FMT, VAR, true>(bits, 0u, a);
    }
    out[j0 + k] = special ? (uint8_t)(Fx<FMT>::NAN_FX >> 24) : (uint8_t)(r >> 24);
  }
}

namespace {

template <int FMT, int VAR>
hipError_t launch_tiles_w(int W, const float* x, uint8_t* out, uint8_t* scales, uint64_t ntiles, int nbits,
                          uint64_t seed, uint64_t blk0, hipStream_t stream) {
  const dim3 grid((unsigned)ntiles), block(kThreads);
#define FBSR_BLOCK_LAUNCH(WW) \
  hipLaunchKernelGGL((block_tiles<FMT, VAR, WW>), grid, block, 0, stream, x, out, scales, nbits, seed, blk0, kXcdLgBlock)
  if constexpr (VAR == kRNE) {
    FBSR_BLOCK_LAUNCH(8);
  } else {
    switch (W) {
      case 1: FBSR_BLOCK_LAUNCH(1); break;
      case 2: FBSR_BLOCK_LAUNCH(2); break;
      case 4: FBSR_BLOCK_LAUNCH(4); break;
      case 8: FBSR_BLOCK_LAUNCH(8); break;
      case 16: FBSR_BLOCK_LAUNCH(16); break;
      default: FBSR_BLOCK_LAUNCH(32); break;
    }
  }
#undef FBSR_BLOCK_LAUNCH
  return hipGetLastError();
}

// Blocks [first element j_from, n) of the call through the per-block kernel; j_from is a multiple of 32.
template <int FMT, int VAR>
hipError_t launch_blocks(const float* x, uint8_t* out, uint8_t* scales, uint64_t j_from, uint64_t n, int nbits, int W,
                         uint64_t seed, uint64_t offset, hipStream_t stream) {
  if (j_from >= n) return hipSuccess;
  const uint64_t m = n - j_from;
  const uint64_t nblk = (m + kScaleBlock - 1) / kScaleBlock;
  for (uint64_t at = 0; at < nblk; at += kMaxElemsPerLaunch) {
    const uint64_t cnt = nblk - at < kMaxElemsPerLaunch ? nblk - at : kMaxElemsPerLaunch;
    const uint64_t e0 = j_from + at * kScaleBlock;
    const uint64_t e_cnt = (at + cnt) * kScaleBlock < m ? cnt * kScaleBlock : m - at * kScaleBlock;
    hipLaunchKernelGGL((block_blocks<FMT, VAR>), dim3((unsigned)((cnt + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       stream, x + e0, out + e0, scales + e0 / kScaleBlock, e_cnt, nbits, W, log2_of(128 / W), seed,
                       offset + e0);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int FMT, int VAR>
hipError_t run(const float* x, uint8_t* out, uint8_t* scales, uint64_t n, int nbits, uint64_t seed, uint64_t offset,
               hipStream_t stream) {
  const int W = VAR == kRNE ? 8 : slot_width(nbits);
  const Split s = split_range(n, offset, W, VAR == kRNE, reinterpret_cast<uintptr_t>(x), 4, 16,
                              reinterpret_cast<uintptr_t>(out), 1, 4);
  // the tile kernel's blocks of 32 must be the call's blocks: it is used only when no head is cut off
  const uint64_t ntiles = s.head == 0 ? s.ntiles : 0;
  for (uint64_t t0 = 0; t0 < ntiles; t0 += kMaxTilesPerLaunch) {
    const uint64_t cnt = ntiles - t0 < kMaxTilesPerLaunch ? ntiles - t0 : kMaxTilesPerLaunch;
    const uint64_t e0 = t0 * s.tile_elems;
    const hipError_t e = launch_tiles_w<FMT, VAR>(W, x + e0, out + e0, scales + e0 / kScaleBlock, cnt, nbits, seed,
                                                  (offset + e0) / (uint64_t)(128 / W), stream);
    if (e != hipSuccess) return e;
  }
  return launch_blocks<FMT, VAR>(x, out, scales, ntiles * s.tile_elems, n, nbits, W, seed, offset, stream);
}

template <int FMT>
hipError_t run_v(int variant, const float* x, uint8_t* out, uint8_t* scales, uint64_t n, int nbits, uint64_t seed,
                 uint64_t offset, hipStream_t stream) {
  switch (variant) {
    case kRNE: return run<FMT, kRNE>(x, out, scales, n, nbits, seed, offset, stream);
    case kSRFF: return run<FMT, kSRFF>(x, out, scales, n, nbits, seed, offset, stream);
    case kSRF: return run<FMT, kSRF>(x, out, scales, n, nbits, seed, offset, stream);
    default: return run<FMT, kSRC>(x, out, scales, n, nbits, seed, offset, stream);
  }
}

}  // namespace

hipError_t launch_round_block_scaled(const float* x, uint8_t* out, uint8_t* scales, uint64_t n, int fmt, int variant,
                                     int nbits, uint64_t seed, uint64_t offset, hipStream_t stream) {
  if (fmt == kE4M3) return run_v<kE4M3>(variant, x, out, scales, n, nbits, seed, offset, stream);
  if (fmt == kE5M2) return run_v<kE5M2>(variant, x, out, scales, n, nbits, seed, offset, stream);
  return run_v<kP4>(variant, x, out, scales, n, nbits, seed, offset, stream);
}

}  // namespace fbsr
