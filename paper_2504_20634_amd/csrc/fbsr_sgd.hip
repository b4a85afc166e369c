// fbsr_sgd.hip -- kernels behind fbsr_sgd_update: the weight update of Alg. 1
// ("w <- RoundTo(w + u), SR applied here") fused into one pass over bf16 weights and fp32
// gradients:  w <- FBSR_bf16(fma(-lr, g, float(w))).
#include "fbsr_launch.h"

namespace fbsr {

// Same workgroup tile as the rounding kernel: per row a lane reads 4 weights (8 bytes) and
// 4 gradients (16 bytes) and writes 4 weights back in place.
template <int VAR, int W>
__global__ __launch_bounds__(kThreads) void sgd_tiles(uint16_t* __restrict__ w, const float* __restrict__ g,
                                                      float neg_lr, int nbits, uint64_t seed, uint64_t step,
                                                      uint64_t blk0, uint32_t xcd_lg) {
  typedef WgTile<W> T;
  __shared__ uint4 strip[T::BLOCKS];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x, xcd_lg);
  const uint64_t row0 = (uint64_t)tile * (T::ELEMS / 4) + (uint64_t)(wave * (kWaveElems / 4) + lane);   // units of 4 elements
  uint64_t* wt = reinterpret_cast<uint64_t*>(w);
  f32x4 gv[kRows];
  uint64_t wv[kRows];
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    gv[k] = load_stream4(g + 4 * (row0 + (uint64_t)(k * 64)));
    wv[k] = wt[row0 + (uint64_t)(k * 64)];   // read-modify-write: keep the line in L2 for the store
  }
  if constexpr (VAR != kRNE) {
    fill_wg_bits<W>(strip, threadIdx.x, blk0 + (uint64_t)tile * T::BLOCKS, seed, step);
    __syncthreads();
  }
  const Addends a = make_addends<kBF16, VAR>(nbits);
  uint32_t b[kRows][4];
  uint32_t umax = 0;
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    const uint32_t lo = (uint32_t)wv[k], hi = (uint32_t)(wv[k] >> 32);
    const float wf[4] = {__uint_as_float(lo << 16), __uint_as_float(lo & 0xFFFF0000u), __uint_as_float(hi << 16),
                         __uint_as_float(hi & 0xFFFF0000u)};
    const float gf[4] = {gv[k].x, gv[k].y, gv[k].z, gv[k].w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      b[k][j] = __float_as_uint(__fmaf_rn(neg_lr, gf[j], wf[j]));
      umax = max(umax, b[k][j] & 0x7FFFFFFFu);
    }
  }
  const bool checked = __any(needs_checked<kBF16>(umax));
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    uint64_t rb = 0;
    if constexpr (VAR != kRNE) rb = read_wg_row_bits<W>(strip, wave, lane, k);
    uint32_t r[4];
    if (checked) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        r[j] = round_pattern<kBF16, VAR, true>(b[k][j], VAR == kRNE ? 0u : slot_bits<W>(rb, j, a.nbits), a);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        r[j] = round_pattern<kBF16, VAR, false>(b[k][j], VAR == kRNE ? 0u : slot_bits<W>(rb, j, a.nbits), a);
    }
    wt[row0 + (uint64_t)(k * 64)] = (uint64_t)pack2_bf16(r[0], r[1]) | ((uint64_t)pack2_bf16(r[2], r[3]) << 32);
  }
}

template <int VAR>
__global__ __launch_bounds__(kThreads) void sgd_elems(uint16_t* __restrict__ w, const float* __restrict__ g,
                                                      uint64_t n, float neg_lr, int nbits, int W, int log2_per_block,
                                                      uint64_t seed, uint64_t step, uint64_t offset) {
  const uint64_t j = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (j >= n) return;
  const Addends a = make_addends<kBF16, VAR>(nbits);
  uint32_t rnd = 0;
  if constexpr (VAR != kRNE) rnd = element_bits(offset + j, log2_per_block, W, a.nbits, seed, step);
  const float x = __fmaf_rn(neg_lr, g[j], __uint_as_float((uint32_t)w[j] << 16));
  w[j] = (uint16_t)(round_pattern<kBF16, VAR, true>(__float_as_uint(x), rnd, a) >> 16);
}

namespace {

template <int VAR, int W>
hipError_t launch_tiles(uint16_t* w, const float* g, uint64_t ntiles, float neg_lr, int nbits, uint64_t seed,
                        uint64_t step, uint64_t blk0, hipStream_t stream) {
  hipLaunchKernelGGL((sgd_tiles<VAR, W>), dim3((unsigned)ntiles), dim3(kThreads), 0, stream, w, g, neg_lr, nbits, seed,
                     step, blk0, kXcdLgSgd);
  return hipGetLastError();
}

template <int VAR>
hipError_t launch_tiles_w(int W, uint16_t* w, const float* g, uint64_t ntiles, float neg_lr, int nbits,
                          uint64_t seed, uint64_t step, uint64_t blk0, hipStream_t stream) {
  if constexpr (VAR == kRNE) return launch_tiles<VAR, 8>(w, g, ntiles, neg_lr, nbits, seed, step, blk0, stream);
  switch (W) {
    case 1: return launch_tiles<VAR, 1>(w, g, ntiles, neg_lr, nbits, seed, step, blk0, stream);
    case 2: return launch_tiles<VAR, 2>(w, g, ntiles, neg_lr, nbits, seed, step, blk0, stream);
    case 4: return launch_tiles<VAR, 4>(w, g, ntiles, neg_lr, nbits, seed, step, blk0, stream);
    case 8: return launch_tiles<VAR, 8>(w, g, ntiles, neg_lr, nbits, seed, step, blk0, stream);
    default: return launch_tiles<VAR, 16>(w, g, ntiles, neg_lr, nbits, seed, step, blk0, stream);
  }
}

template <int VAR>
hipError_t run(uint16_t* w, const float* g, uint64_t n, float neg_lr, int nbits, uint64_t seed, uint64_t step,
               uint64_t offset, hipStream_t stream) {
  const int W = VAR == kRNE ? 8 : slot_width(nbits);
  const Split s = split_range(n, offset, W, VAR == kRNE, reinterpret_cast<uintptr_t>(g), 4, 16,
                              reinterpret_cast<uintptr_t>(w), 2, 8);
  return run_split(
      s, n,
      [&](uint64_t first, uint64_t count) {
        hipLaunchKernelGGL((sgd_elems<VAR>), elems_grid(count), dim3(kThreads), 0, stream, w + first, g + first, count, neg_lr,
                           nbits, W, log2_of(128 / W), seed, step, offset + first);
        return hipGetLastError();
      },
      [&](uint64_t first, uint64_t count) {
        return launch_tiles_w<VAR>(W, w + first, g + first, count, neg_lr, nbits, seed, step,
                                   (offset + first) / (uint64_t)(128 / W), stream);
      });
}

}  // namespace

hipError_t launch_sgd(void* w, const float* g, uint64_t n, float lr, int variant, int nbits, uint64_t seed,
                      uint64_t step, uint64_t offset, hipStream_t stream) {
  uint16_t* wp = reinterpret_cast<uint16_t*>(w);
  const float neg_lr = -lr;
  switch (variant) {
    case kRNE: return run<kRNE>(wp, g, n, neg_lr, nbits, seed, step, offset, stream);
    case kSRFF: return run<kSRFF>(wp, g, n, neg_lr, nbits, seed, step, offset, stream);
    case kSRF: return run<kSRF>(wp, g, n, neg_lr, nbits, seed, step, offset, stream);
    default: return run<kSRC>(wp, g, n, neg_lr, nbits, seed, step, offset, stream);
  }
}

}  // namespace fbsr
