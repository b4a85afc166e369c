// fbsr_round.hip -- kernels behind fbsr_round: fp32 -> {bf16, E4M3, E5M2} few-bit stochastic
// rounding (Sec. II-B SRFF / SRF, Eq. (7) SRC, Sec. II-A RNE).
#include "fbsr_launch.h"

namespace fbsr {

// One workgroup of RoundGeometry<FMT>::WAVES waves per tile (8 and 4096 elements for the 8-bit targets, 4 and 2048 for
// bf16), one wave per 512 elements.  Streaming: every input byte
// is read once (16-byte loads, fully coalesced: a row of 256 floats per load instruction) and
// every output byte written once (4 bytes per lane for fp8, 8 for bf16).  The loads are issued
// first so that their latency overlaps the Philox rounds.
template <int FMT, int VAR, int W>
__global__ __launch_bounds__(RoundGeometry<FMT>::THREADS) void round_tiles(const float* __restrict__ x, void* __restrict__ out,
                                                                            int nbits, uint64_t seed, uint64_t blk0,
                                                                            uint32_t xcd_lg) {
  typedef WgTile<W, RoundGeometry<FMT>::WAVES> T;
  __shared__ uint4 strip[T::BLOCKS];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x, xcd_lg);
  const uint64_t row0 = (uint64_t)tile * (T::ELEMS / 4) + (uint64_t)(wave * (kWaveElems / 4) + lane);   // units of 4 elements
  f32x4 v[kRows];
#pragma unroll
  for (int k = 0; k < kRows; ++k) v[k] = load_stream4(x + 4 * (row0 + (uint64_t)(k * 64)));
  if constexpr (VAR != kRNE) {
    fill_wg_bits<W, RoundGeometry<FMT>::WAVES>(strip, threadIdx.x, blk0 + (uint64_t)tile * T::BLOCKS, seed, 0);
    __syncthreads();
  }
  // W = 32: more than 16 random bits, one 32-bit slot per element (a row's four slots are one Philox block).  The fp8
  // targets still go through the hardware converts, which take a random operand of 32 bits; only a wave that holds a
  // NaN, and bf16, take the integer arithmetic, in its flavour for many bits.
  constexpr bool MANY = W == 32;
  const Addends a = make_addends<FMT, VAR>(MANY ? kMaxTileNbits : nbits);
  ManyAddends many = {a, 0.0f};
  if constexpr (MANY && VAR != kRNE) many = make_many_addends<FMT, VAR>(nbits);
  HwAddends hw = {0, 0, 0, 0};
  if constexpr (Fx<FMT>::kIsFp8 && VAR != kRNE) hw = make_hw_addends<FMT, VAR>(nbits);
  uint32_t umax = 0;
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    umax = max(umax, max(max(__float_as_uint(v[k].x) & 0x7FFFFFFFu, __float_as_uint(v[k].y) & 0x7FFFFFFFu),
                         max(__float_as_uint(v[k].z) & 0x7FFFFFFFu, __float_as_uint(v[k].w) & 0x7FFFFFFFu)));
  }
  const bool checked = __any(needs_checked<FMT>(umax));   // wave-uniform: NaN (bf16: also |x| > M) is rare
  // with more random bits than the hardware converts apply exactly to every input, a wave that holds a non-zero value
  // below the target's normal range takes the integer arithmetic
  bool hw_ok = true;
  if constexpr (MANY && Fx<FMT>::kIsFp8) {
    if (hw_needs_normal_inputs<FMT, VAR>(nbits)) {   // uniform over the launch
      uint32_t lowest = 0xFFFFFFFFu;
#pragma unroll
      for (int k = 0; k < kRows; ++k)
        lowest = min(lowest, min(min(magnitude_less_one(__float_as_uint(v[k].x)), magnitude_less_one(__float_as_uint(v[k].y))),
                                 min(magnitude_less_one(__float_as_uint(v[k].z)), magnitude_less_one(__float_as_uint(v[k].w)))));
      hw_ok = !__any(lowest < Fx<FMT>::U_SUB - 1u);
    }
  }
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    uint32_t n4[4] = {0, 0, 0, 0};
    if constexpr (VAR != kRNE) row_draws4<W>(strip, wave, lane, k, (uint32_t)nbits, n4);
    const uint32_t b[4] = {__float_as_uint(v[k].x), __float_as_uint(v[k].y), __float_as_uint(v[k].z),
                           __float_as_uint(v[k].w)};
    const uint64_t row = row0 + (uint64_t)(k * 64);
    if constexpr (Fx<FMT>::kIsFp8 && VAR != kRNE) {
      if (!checked && hw_ok) {   // no NaN among the wave's elements: the hardware converts apply
        __builtin_nontemporal_store(round4_fp8_hw<FMT, VAR, MANY>(b, n4, hw), reinterpret_cast<uint32_t*>(out) + row);
        continue;
      }
    }
    uint32_t r[4];
    if constexpr (MANY && VAR != kRNE) {
      if (checked) {
#pragma unroll
        for (int j = 0; j < 4; ++j) r[j] = round_pattern_many<FMT, VAR, true>(b[j], n4[j], (uint32_t)nbits, many);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) r[j] = round_pattern_many<FMT, VAR, false>(b[j], n4[j], (uint32_t)nbits, many);
      }
    } else if (checked) {
#pragma unroll
      for (int j = 0; j < 4; ++j) r[j] = round_pattern<FMT, VAR, true>(b[j], n4[j], a);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) r[j] = round_pattern<FMT, VAR, false>(b[j], n4[j], a);
    }
    if constexpr (Fx<FMT>::kIsFp8) {
      __builtin_nontemporal_store(pack4_fp8<FMT>(r[0], r[1], r[2], r[3]), reinterpret_cast<uint32_t*>(out) + row);
    } else {
      const uint64_t pv = (uint64_t)pack2_bf16(r[0], r[1]) | ((uint64_t)pack2_bf16(r[2], r[3]) << 32);
      __builtin_nontemporal_store(pv, reinterpret_cast<uint64_t*>(out) + row);
    }
  }
}

// One thread per element: any alignment, any offset, ragged heads and tails.  Each thread
// computes the whole Philox block its element lives in.
template <int FMT, int VAR>
__global__ __launch_bounds__(kThreads) void round_elems(const float* __restrict__ x, void* __restrict__ out,
                                                        uint64_t n, int nbits, int W, int log2_per_block,
                                                        uint64_t seed, uint64_t offset) {
  const uint64_t j = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (j >= n) return;
  uint32_t r;
  if constexpr (VAR != kRNE) {
    const uint32_t rnd = element_bits(offset + j, log2_per_block, W, (uint32_t)nbits, seed, 0);
    if (nbits > kMaxTileNbits) r = round_pattern_wide<FMT, VAR>(__float_as_uint(x[j]), rnd, (uint32_t)nbits);   // uniform over the launch
    else r = round_pattern<FMT, VAR, true>(__float_as_uint(x[j]), rnd, make_addends<FMT, VAR>(nbits));
  } else {
    r = round_pattern<FMT, VAR, true>(__float_as_uint(x[j]), 0u, make_addends<FMT, VAR>(nbits));
  }
  typedef typename Fx<FMT>::code_t code_t;
  reinterpret_cast<code_t*>(out)[j] = (code_t)(r >> Fx<FMT>::FRAC);
}

// Measurement aid: the same tile geometry with no arithmetic -- every float is read once (16-byte loads) and
// its top byte written (4-byte stores), a plain 4 : 1 read : write stream.  What this reaches is the practical
// ceiling of the rounding kernels' launch shape on the part at hand.
__global__ __launch_bounds__(kRoundThreads) void stream41_tiles(const float* __restrict__ x, uint8_t* __restrict__ out, uint32_t xcd_lg) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x, xcd_lg);
  const uint64_t row0 = (uint64_t)tile * (kRoundTileElems / 4) + (uint64_t)(wave * (kWaveElems / 4) + lane);
  f32x4 v[kRows];
#pragma unroll
  for (int k = 0; k < kRows; ++k) v[k] = load_stream4(x + 4 * (row0 + (uint64_t)(k * 64)));
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    const uint32_t packed = pack4_fp8<kE4M3>(__float_as_uint(v[k].x), __float_as_uint(v[k].y), __float_as_uint(v[k].z),
                                             __float_as_uint(v[k].w));
    __builtin_nontemporal_store(packed, reinterpret_cast<uint32_t*>(out) + row0 + (uint64_t)(k * 64));
  }
}

hipError_t launch_stream41(const float* x, uint8_t* out, uint64_t ntiles, hipStream_t stream) {
  return in_pieces(ntiles, kMaxTilesPerLaunch, [&](uint64_t t0, uint64_t count) {
    hipLaunchKernelGGL(stream41_tiles, dim3((unsigned)count), dim3(kRoundThreads), 0, stream, x + t0 * kRoundTileElems,
                       out + t0 * kRoundTileElems, kXcdLgRound);
    return hipGetLastError();
  });
}

namespace {

template <int FMT, int VAR, int W>
hipError_t launch_tiles(const float* x, void* out, uint64_t ntiles, int nbits, uint64_t seed, uint64_t blk0,
                        hipStream_t stream) {
  hipLaunchKernelGGL((round_tiles<FMT, VAR, W>), dim3((unsigned)ntiles), dim3(RoundGeometry<FMT>::THREADS), 0, stream, x, out,
                     nbits, seed, blk0, RoundGeometry<FMT>::XCD_LG);
  return hipGetLastError();
}

template <int FMT, int VAR>
hipError_t launch_tiles_w(int W, const float* x, void* out, uint64_t ntiles, int nbits, uint64_t seed,
                          uint64_t blk0, hipStream_t stream) {
  if constexpr (VAR == kRNE) {
    return launch_tiles<FMT, VAR, 8>(x, out, ntiles, nbits, seed, blk0, stream);
  } else {
    switch (W) {
      case 1: return launch_tiles<FMT, VAR, 1>(x, out, ntiles, nbits, seed, blk0, stream);
      case 2: return launch_tiles<FMT, VAR, 2>(x, out, ntiles, nbits, seed, blk0, stream);
      case 4: return launch_tiles<FMT, VAR, 4>(x, out, ntiles, nbits, seed, blk0, stream);
      case 8: return launch_tiles<FMT, VAR, 8>(x, out, ntiles, nbits, seed, blk0, stream);
      case 16: return launch_tiles<FMT, VAR, 16>(x, out, ntiles, nbits, seed, blk0, stream);
      default: return launch_tiles<FMT, VAR, 32>(x, out, ntiles, nbits, seed, blk0, stream);
    }
  }
}

template <int FMT, int VAR>
hipError_t run(const float* x, void* out, uint64_t n, int nbits, uint64_t seed, uint64_t offset,
               hipStream_t stream) {
  const int W = VAR == kRNE ? 8 : slot_width(nbits);
  const uint64_t osize = sizeof(typename Fx<FMT>::code_t);
  const Split s = split_range(n, offset, W, VAR == kRNE, reinterpret_cast<uintptr_t>(x), 4, 16,
                              reinterpret_cast<uintptr_t>(out), osize, 4 * osize, 0, 0, 1, RoundGeometry<FMT>::TILE_ELEMS);
  char* o = reinterpret_cast<char*>(out);
  return run_split(
      s, n,
      [&](uint64_t first, uint64_t count) {
        hipLaunchKernelGGL((round_elems<FMT, VAR>), elems_grid(count), dim3(kThreads), 0, stream, x + first,
                           reinterpret_cast<void*>(o + first * osize), count, nbits, W, log2_of(128 / W), seed, offset + first);
        return hipGetLastError();
      },
      [&](uint64_t first, uint64_t count) {
        return launch_tiles_w<FMT, VAR>(W, x + first, o + first * osize, count, nbits, seed,
                                        (offset + first) / (uint64_t)(128 / W), stream);
      });
}

template <int FMT>
hipError_t run_v(int variant, const float* x, void* out, uint64_t n, int nbits, uint64_t seed, uint64_t offset,
                 hipStream_t stream) {
  switch (variant) {
    case kRNE: return run<FMT, kRNE>(x, out, n, nbits, seed, offset, stream);
    case kSRFF: return run<FMT, kSRFF>(x, out, n, nbits, seed, offset, stream);
    case kSRF: return run<FMT, kSRF>(x, out, n, nbits, seed, offset, stream);
    default: return run<FMT, kSRC>(x, out, n, nbits, seed, offset, stream);
  }
}

}  // namespace

hipError_t launch_round(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
                        uint64_t offset, hipStream_t stream) {
  switch (fmt) {
    case kBF16: return run_v<kBF16>(variant, x, out, n, nbits, seed, offset, stream);
    case kE4M3: return run_v<kE4M3>(variant, x, out, n, nbits, seed, offset, stream);
    case kE5M2: return run_v<kE5M2>(variant, x, out, n, nbits, seed, offset, stream);
    default: return run_v<kP4>(variant, x, out, n, nbits, seed, offset, stream);
  }
}

}  // namespace fbsr
