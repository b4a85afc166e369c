// fbsr_round16.hip -- kernels behind fbsr_round_from16: bf16 / IEEE binary16 -> {E4M3, E5M2} few-bit
// stochastic rounding, the narrow-source setting of Sec. III-E and Fig. 2 (few excess bits D).
// The source value is widened exactly to an fp32 pattern and then takes the same rounding core as
// fbsr_round.
#include "fbsr_launch.h"

namespace fbsr {

// One workgroup per PAIR of consecutive 2048-element tiles; per tile one wave takes 512 elements, a lane one
// 16-byte load of 8 source codes and one 8-byte store of 8 fp8 codes: 3 bytes of traffic per element.  At 3 bytes
// per element a single tile is only 6 KiB of traffic per workgroup; measured on a plain 2 : 1 stream of 2^28
// elements, 4096 elements per workgroup reach 6.65 TB/s (with runs of 128 workgroups per XCD) where 2048 reach
// 6.05-6.35 and 8192 6.3-6.5.  Both tiles' loads are issued first, and the pair's Philox blocks are dealt to the
// threads together.  `ntiles` is the number of tiles of the launch; an odd one leaves the last workgroup one tile.
constexpr int kPair16 = 2;

template <int SRC, int FMT, int VAR, int W>
__global__ __launch_bounds__(kThreads) void round16_tiles(const uint16_t* __restrict__ x, uint8_t* __restrict__ out,
                                                          uint32_t ntiles, int nbits, uint64_t seed, uint64_t blk0,
                                                          uint32_t xcd_lg) {
  typedef WgTile<W> T;
  __shared__ uint4 strip[kPair16 * T::BLOCKS];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int e0 = wave * kWaveElems + 8 * lane;                                  // tile-relative first element
  const uint32_t tile0 = xcd_tile(blockIdx.x, gridDim.x, xcd_lg) * kPair16;     // < ntiles: one workgroup per started pair
  const int here = ntiles - tile0 < (uint32_t)kPair16 ? (int)(ntiles - tile0) : kPair16;
  u32x4 q[kPair16];
#pragma unroll
  for (int t = 0; t < kPair16; ++t)
    if (t < here) q[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + ((uint64_t)(tile0 + t) * T::ELEMS + (uint64_t)e0)));
  if constexpr (VAR != kRNE) {
    for (int bi = threadIdx.x; bi < here * T::BLOCKS; bi += kThreads) {
      uint32_t o[4];
      philox_block(blk0 + (uint64_t)tile0 * T::BLOCKS + (uint64_t)bi, seed, 0, o);
      strip[bi] = make_uint4(o[0], o[1], o[2], o[3]);
    }
    __syncthreads();
  }
  constexpr bool MANY = W == 32;   // more than 16 random bits: 32-bit slots
  const Addends a = make_addends<FMT, VAR>(MANY ? kMaxTileNbits : nbits);
  ManyAddends many = {a, 0.0f};
  if constexpr (MANY && VAR != kRNE) many = make_many_addends<FMT, VAR>(nbits);
  HwAddends hw = {0, 0, 0, 0};
  if constexpr (VAR != kRNE) hw = make_hw_addends<FMT, VAR>(nbits);
#pragma unroll
  for (int t = 0; t < kPair16; ++t) {
    if (t >= here) break;   // uniform over the workgroup
    const uint32_t words[4] = {q[t].x, q[t].y, q[t].z, q[t].w};
    uint32_t b[8];
    uint32_t umax = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      b[j] = widen16<SRC>((words[j >> 1] >> (16 * (j & 1))) & 0xFFFFu);
      umax = max(umax, b[j] & 0x7FFFFFFFu);
    }
    bool checked = __any(needs_checked<FMT>(umax));   // wave-uniform: a NaN among the wave's elements
    if constexpr (MANY) {
      // more random bits than the hardware converts apply exactly to every input: they serve a wave only if it holds no
      // non-zero value below the target's normal range
      if (hw_needs_normal_inputs<FMT, VAR>(nbits)) {
        uint32_t lowest = 0xFFFFFFFFu;
#pragma unroll
        for (int j = 0; j < 8; ++j) lowest = min(lowest, magnitude_less_one(b[j]));
        checked = checked || __any(lowest < Fx<FMT>::U_SUB - 1u);
      }
    }
    uint32_t n[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (VAR != kRNE) read_wg_bits8<W>(strip + t * T::BLOCKS, e0, (uint32_t)nbits, n);
    uint32_t packed[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t b4[4] = {b[4 * h], b[4 * h + 1], b[4 * h + 2], b[4 * h + 3]};
      const uint32_t n4[4] = {n[4 * h], n[4 * h + 1], n[4 * h + 2], n[4 * h + 3]};
      bool done = false;
      if constexpr (VAR != kRNE) {
        if (!checked) {
          packed[h] = round4_fp8_hw<FMT, VAR, MANY>(b4, n4, hw);
          done = true;
        }
      }
      if (!done) {
        uint32_t r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if constexpr (MANY && VAR != kRNE) r[j] = round_pattern_many<FMT, VAR, true>(b4[j], n4[j], (uint32_t)nbits, many);
          else r[j] = round_pattern<FMT, VAR, true>(b4[j], n4[j], a);
        }
        packed[h] = pack4_fp8<FMT>(r[0], r[1], r[2], r[3]);
      }
    }
    __builtin_nontemporal_store((uint64_t)packed[0] | ((uint64_t)packed[1] << 32),
                                reinterpret_cast<uint64_t*>(out + ((uint64_t)(tile0 + t) * T::ELEMS + (uint64_t)e0)));
  }
}

template <int SRC, int FMT, int VAR>
__global__ __launch_bounds__(kThreads) void round16_elems(const uint16_t* __restrict__ x, uint8_t* __restrict__ out,
                                                          uint64_t n, int nbits, int W, int log2_per_block,
                                                          uint64_t seed, uint64_t offset) {
  const uint64_t j = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (j >= n) return;
  uint32_t r;
  if constexpr (VAR != kRNE) {
    const uint32_t rnd = element_bits(offset + j, log2_per_block, W, (uint32_t)nbits, seed, 0);
    if (nbits > kMaxTileNbits) r = round_pattern_wide<FMT, VAR>(widen16<SRC>(x[j]), rnd, (uint32_t)nbits);   // uniform over the launch
    else r = round_pattern<FMT, VAR, true>(widen16<SRC>(x[j]), rnd, make_addends<FMT, VAR>(nbits));
  } else {
    r = round_pattern<FMT, VAR, true>(widen16<SRC>(x[j]), 0u, make_addends<FMT, VAR>(nbits));
  }
  out[j] = (uint8_t)(r >> Fx<FMT>::FRAC);
}

namespace {

template <int SRC, int FMT, int VAR>
hipError_t launch_tiles_w(int W, const uint16_t* x, uint8_t* out, uint64_t ntiles, int nbits, uint64_t seed,
                          uint64_t blk0, hipStream_t stream) {
  const dim3 grid((unsigned)((ntiles + kPair16 - 1) / kPair16)), block(kThreads);
  if constexpr (VAR == kRNE) {
    hipLaunchKernelGGL((round16_tiles<SRC, FMT, VAR, 8>), grid, block, 0, stream, x, out, (uint32_t)ntiles, nbits, seed, blk0, kXcdLgRound16);
  } else {
    switch (W) {
      case 1: hipLaunchKernelGGL((round16_tiles<SRC, FMT, VAR, 1>), grid, block, 0, stream, x, out, (uint32_t)ntiles, nbits, seed, blk0, kXcdLgRound16); break;
      case 2: hipLaunchKernelGGL((round16_tiles<SRC, FMT, VAR, 2>), grid, block, 0, stream, x, out, (uint32_t)ntiles, nbits, seed, blk0, kXcdLgRound16); break;
      case 4: hipLaunchKernelGGL((round16_tiles<SRC, FMT, VAR, 4>), grid, block, 0, stream, x, out, (uint32_t)ntiles, nbits, seed, blk0, kXcdLgRound16); break;
      case 8: hipLaunchKernelGGL((round16_tiles<SRC, FMT, VAR, 8>), grid, block, 0, stream, x, out, (uint32_t)ntiles, nbits, seed, blk0, kXcdLgRound16); break;
      case 16: hipLaunchKernelGGL((round16_tiles<SRC, FMT, VAR, 16>), grid, block, 0, stream, x, out, (uint32_t)ntiles, nbits, seed, blk0, kXcdLgRound16); break;
      default: hipLaunchKernelGGL((round16_tiles<SRC, FMT, VAR, 32>), grid, block, 0, stream, x, out, (uint32_t)ntiles, nbits, seed, blk0, kXcdLgRound16); break;
    }
  }
  return hipGetLastError();
}

template <int SRC, int FMT, int VAR>
hipError_t run(const uint16_t* x, uint8_t* out, uint64_t n, int nbits, uint64_t seed, uint64_t offset,
               hipStream_t stream) {
  const int W = VAR == kRNE ? 8 : slot_width(nbits);
  const Split s = split_range(n, offset, W, VAR == kRNE, reinterpret_cast<uintptr_t>(x), 2, 16,
                              reinterpret_cast<uintptr_t>(out), 1, 8);
  return run_split(
      s, n,
      [&](uint64_t first, uint64_t count) {
        hipLaunchKernelGGL((round16_elems<SRC, FMT, VAR>), elems_grid(count), dim3(kThreads), 0, stream, x + first, out + first,
                           count, nbits, W, log2_of(128 / W), seed, offset + first);
        return hipGetLastError();
      },
      [&](uint64_t first, uint64_t count) {
        return launch_tiles_w<SRC, FMT, VAR>(W, x + first, out + first, count, nbits, seed,
                                             (offset + first) / (uint64_t)(128 / W), stream);
      });
}

template <int SRC, int FMT>
hipError_t run_v(int variant, const uint16_t* x, uint8_t* out, uint64_t n, int nbits, uint64_t seed, uint64_t offset,
                 hipStream_t stream) {
  switch (variant) {
    case kRNE: return run<SRC, FMT, kRNE>(x, out, n, nbits, seed, offset, stream);
    case kSRFF: return run<SRC, FMT, kSRFF>(x, out, n, nbits, seed, offset, stream);
    case kSRF: return run<SRC, FMT, kSRF>(x, out, n, nbits, seed, offset, stream);
    default: return run<SRC, FMT, kSRC>(x, out, n, nbits, seed, offset, stream);
  }
}

template <int SRC>
hipError_t run_f(int fmt, int variant, const uint16_t* x, uint8_t* out, uint64_t n, int nbits, uint64_t seed,
                 uint64_t offset, hipStream_t stream) {
  if (fmt == kE4M3) return run_v<SRC, kE4M3>(variant, x, out, n, nbits, seed, offset, stream);
  if (fmt == kE5M2) return run_v<SRC, kE5M2>(variant, x, out, n, nbits, seed, offset, stream);
  return run_v<SRC, kP4>(variant, x, out, n, nbits, seed, offset, stream);
}

}  // namespace

hipError_t launch_round_from16(const void* x, void* out, uint64_t n, int src_fmt, int fmt, int variant, int nbits,
                               uint64_t seed, uint64_t offset, hipStream_t stream) {
  const uint16_t* xp = reinterpret_cast<const uint16_t*>(x);
  uint8_t* op = reinterpret_cast<uint8_t*>(out);
  if (src_fmt == kSrcBF16) return run_f<kSrcBF16>(fmt, variant, xp, op, n, nbits, seed, offset, stream);
  return run_f<kSrcFP16>(fmt, variant, xp, op, n, nbits, seed, offset, stream);
}

}  // namespace fbsr
