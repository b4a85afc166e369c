// fbsr_stats.hip -- kernels behind fbsr_bias_stats: round as fbsr_round and reduce, per bin,
// {count, sum y, sum e, sum e^2} with y the decoded rounded value and e = (y - x) / ulp_t(x)
// in fp64 -- the measurement behind Figs. 1 and 2 (mean rounded value per input, bias in
// target ulps, Sec. III).  Bins are runs of `group` consecutive global indices.
//
// Reduction order is fixed (lane-local sums -> xor-butterfly across the wave -> one record
// per tile in the workspace -> per-bin sums over its tiles, lane-strided then butterfly), so
// results are bit-reproducible; no floating-point atomics are used.
#include "fbsr_launch.h"

namespace fbsr {

struct Acc {
  double sy, se, see;
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
  const int ef = (int)((bits >> 23) & 0xFFu) - 127;
  const int et = ef > 1 - F::B ? ef : 1 - F::B;
  const uint32_t hi = (uint32_t)(1023 + F::P - 1 - et) << 20;
  return __hiloint2double((int)hi, 0);
}

template <int FMT>
__device__ __forceinline__ void accumulate(Acc& acc, uint32_t bits, uint32_t r) {
  const double y = (double)decode_top<FMT>(r);
  const double e = (y - (double)__uint_as_float(bits)) * inv_ulp<FMT>(bits);
  acc.sy += y;
  acc.se += e;
  acc.see = fma(e, e, acc.see);
}

// Same workgroup tile as the rounding kernel.  A tile touches at most two bins (the host
// guarantees group >= tile): lane-local fp64 sums for the first (A) and second (B) bin, an
// xor-butterfly across each wave, the four waves' sums staged in LDS and added in wave order,
// one record per tile = {A.sy, A.se, A.see, B.sy, B.se, B.see}.
template <int FMT, int VAR, int W>
__global__ __launch_bounds__(kThreads) void stats_tiles(const float* __restrict__ x, void* __restrict__ out, int nbits,
                                                        uint64_t seed, uint64_t blk0, uint64_t i0, uint64_t group,
                                                        double* __restrict__ records) {
  typedef WgTile<W> T;
  __shared__ uint4 strip[T::BLOCKS];
  __shared__ double staged[kWavesPerBlock][kStatsRecordDoubles];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const uint64_t row0 = (uint64_t)blockIdx.x * (T::ELEMS / 4) + (uint64_t)(wave * (kWaveElems / 4) + lane);   // units of 4 elements
  f32x4 v[kRows];
#pragma unroll
  for (int k = 0; k < kRows; ++k) v[k] = load_stream4(x + 4 * (row0 + (uint64_t)(k * 64)));
  if constexpr (VAR != kRNE) {
    fill_wg_bits<W>(strip, threadIdx.x, blk0 + (uint64_t)blockIdx.x * T::BLOCKS, seed, 0);
    __syncthreads();
  }
  const Addends a = make_addends<FMT, VAR>(nbits);
  const uint64_t gi0 = i0 + (uint64_t)blockIdx.x * T::ELEMS;   // global index of the tile's first element
  const uint64_t to_boundary = group - gi0 % group;           // tile-relative index where the second bin starts
  const int boundary = to_boundary > (uint64_t)T::ELEMS ? T::ELEMS : (int)to_boundary;
  Acc accA = {0.0, 0.0, 0.0}, accB = {0.0, 0.0, 0.0};
  uint32_t r[kRows][4], b[kRows][4];
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    uint64_t rb = 0;
    if constexpr (VAR != kRNE) rb = read_wg_row_bits<W>(strip, wave, lane, k);
    b[k][0] = __float_as_uint(v[k].x); b[k][1] = __float_as_uint(v[k].y);
    b[k][2] = __float_as_uint(v[k].z); b[k][3] = __float_as_uint(v[k].w);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      r[k][j] = round_pattern<FMT, VAR, true>(b[k][j], VAR == kRNE ? 0u : slot_bits<W>(rb, j, a.nbits), a);
    if (out != nullptr) {
      const uint64_t row = row0 + (uint64_t)(k * 64);
      if constexpr (Fx<FMT>::kIsFp8) {
        reinterpret_cast<uint32_t*>(out)[row] = pack4_fp8<FMT>(r[k][0], r[k][1], r[k][2], r[k][3]);
      } else {
        reinterpret_cast<uint64_t*>(out)[row] =
            (uint64_t)pack2_bf16(r[k][0], r[k][1]) | ((uint64_t)pack2_bf16(r[k][2], r[k][3]) << 32);
      }
    }
  }
  const int w_lo = wave * kWaveElems, w_hi = w_lo + kWaveElems;   // this wave's tile-relative range
  if (boundary >= w_hi) {            // the whole wave lies in the first bin (wave-uniform, the common case)
#pragma unroll
    for (int k = 0; k < kRows; ++k)
#pragma unroll
      for (int j = 0; j < 4; ++j) accumulate<FMT>(accA, b[k][j], r[k][j]);
  } else if (boundary <= w_lo) {     // the whole wave lies in the second bin
#pragma unroll
    for (int k = 0; k < kRows; ++k)
#pragma unroll
      for (int j = 0; j < 4; ++j) accumulate<FMT>(accB, b[k][j], r[k][j]);
  } else {                           // the bin boundary falls inside this wave's elements
#pragma unroll
    for (int k = 0; k < kRows; ++k)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int e = w_lo + k * 256 + 4 * lane + j;
        if (e < boundary) accumulate<FMT>(accA, b[k][j], r[k][j]);
        else accumulate<FMT>(accB, b[k][j], r[k][j]);
      }
  }
  const double s0 = wave_sum(accA.sy), s1 = wave_sum(accA.se), s2 = wave_sum(accA.see);
  const double s3 = wave_sum(accB.sy), s4 = wave_sum(accB.se), s5 = wave_sum(accB.see);
  if (lane == 0) {
    staged[wave][0] = s0; staged[wave][1] = s1; staged[wave][2] = s2;
    staged[wave][3] = s3; staged[wave][4] = s4; staged[wave][5] = s5;
  }
  __syncthreads();
  if (threadIdx.x < kStatsRecordDoubles) {
    double t = staged[0][threadIdx.x];
#pragma unroll
    for (int wv = 1; wv < kWavesPerBlock; ++wv) t += staged[wv][threadIdx.x];
    records[(uint64_t)blockIdx.x * kStatsRecordDoubles + threadIdx.x] = t;
  }
}

// One wave per bin: sums the records of the tiles that overlap the bin and adds the bin's
// totals to the caller's statistics.  Tiles cover global indices [i0, i0 + ntiles * tile_elems).
__global__ __launch_bounds__(64) void stats_finalize(const double* __restrict__ records, uint64_t ntiles,
                                                     uint64_t tile_elems, uint64_t i0, uint64_t group,
                                                     uint64_t bin_lo, uint64_t first_bin, double* __restrict__ stats) {
  const int lane = threadIdx.x;
  const uint64_t bin = bin_lo + blockIdx.x;
  const uint64_t i_end = i0 + ntiles * tile_elems;
  const uint64_t lo = bin * group > i0 ? bin * group : i0;
  const uint64_t hi = (bin + 1) * group < i_end ? (bin + 1) * group : i_end;
  if (lo >= hi) return;
  const uint64_t t_lo = (lo - i0) / tile_elems, t_hi = (hi - 1 - i0) / tile_elems;
  double sy = 0.0, se = 0.0, see = 0.0;
  for (uint64_t t = t_lo + (uint64_t)lane; t <= t_hi; t += 64) {
    // the tile's first bin is this bin iff the tile starts inside it
    const double* rec = records + t * kStatsRecordDoubles + ((i0 + t * tile_elems >= bin * group) ? 0 : 3);
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
  const Addends a = make_addends<FMT, VAR>(nbits);
  Acc acc = {0.0, 0.0, 0.0};
  typedef typename Fx<FMT>::code_t code_t;
  for (uint64_t i = lo; i < hi; ++i) {
    uint32_t rnd = 0;
    if constexpr (VAR != kRNE) rnd = element_bits(i, log2_per_block, W, a.nbits, seed, 0);
    const uint32_t bits = __float_as_uint(x[i - a0]);
    const uint32_t r = round_pattern<FMT, VAR, true>(bits, rnd, a);
    if (out != nullptr) reinterpret_cast<code_t*>(out)[i - a0] = (code_t)(r >> Fx<FMT>::FRAC);
    accumulate<FMT>(acc, bits, r);
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
  hipLaunchKernelGGL((stats_tiles<FMT, VAR, W>), dim3((unsigned)ntiles), dim3(kThreads), 0, stream, x, out, nbits, seed,
                     blk0, i0, group, records);
  return hipGetLastError();
}

template <int FMT, int VAR>
hipError_t launch_tiles_w(int W, const float* x, void* out, uint64_t ntiles, int nbits, uint64_t seed,
                          uint64_t blk0, uint64_t i0, uint64_t group, double* records, hipStream_t stream) {
  if constexpr (VAR == kRNE) return launch_tiles<FMT, VAR, 8>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
  switch (W) {
    case 1: return launch_tiles<FMT, VAR, 1>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
    case 2: return launch_tiles<FMT, VAR, 2>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
    case 4: return launch_tiles<FMT, VAR, 4>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
    case 8: return launch_tiles<FMT, VAR, 8>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
    default: return launch_tiles<FMT, VAR, 16>(x, out, ntiles, nbits, seed, blk0, i0, group, records, stream);
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
    hipLaunchKernelGGL(stats_finalize, dim3((unsigned)(bin_hi - bin_lo + 1)), dim3(64), 0, stream, workspace, s.ntiles,
                       s.tile_elems, i0, group, bin_lo, first_bin, stats);
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

hipError_t launch_stats(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
                        uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins, double* stats,
                        double* workspace, hipStream_t stream) {
  (void)nbins;
  switch (fmt) {
    case kBF16: return run_v<kBF16>(variant, x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
    case kE4M3: return run_v<kE4M3>(variant, x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
    default: return run_v<kE5M2>(variant, x, out, n, nbits, seed, offset, group, first_bin, stats, workspace, stream);
  }
}

}  // namespace fbsr
