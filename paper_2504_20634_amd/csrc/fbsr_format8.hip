// fbsr_format8.hip -- kernels behind fbsr_round_format8 and fbsr_round_format16: few-bit stochastic rounding of
// fp32 / bf16 / binary16 values to ANY format (K, P, B; M) of Sec. II, Eq. (1) with K <= 8 (one code per byte) or
// K <= 16 (one code per 16-bit word; the code space then has 32 - K fraction bits), plus the deterministic
// modes of Sec. II-A (nearest with ties to even, to odd, away from zero) and Eq. (7) with either tie
// rule for its inner rounding (Sec. III-F).
//
// The arithmetic is the code-space addition of fbsr_device.h with the format's constants as
// wave-uniform kernel arguments instead of template parameters: a 32-bit word whose top byte is the
// magnitude code and whose low 24 bits are delta 2^24; every predicate is one integer addition.
//     nearest-even   + 2^23 - 1 + (last kept bit)          ties-to-odd   + 2^23 - 1 + (last kept bit ^ 1)
//     ties-away      + 2^23                                 SRFF / SRF / SRC as in fbsr_device.h
// Above M a format with an infinity takes the nearest-even addend of M's own parity, which carries
// into the code after max_code; that code is then replaced by the infinity's.
#include <mutex>

#include "fbsr_launch.h"

namespace fbsr {

// One workgroup per 2048-element tile, one wave per 512 elements.  fp32 source: two rows of 256
// elements per wave, a lane owns 4 consecutive floats per row (16-byte load, 4-byte store).  16-bit
// sources: a lane owns 8 consecutive codes (16-byte load, 8-byte store).  W = 0: the mode draws no bits.
// WIDE: 16-bit codes (a lane then stores 8 bytes per row of an fp32 source, 16 bytes from a 16-bit source).
template <int SRC, bool TIES, int W, bool WIDE>
__global__ __launch_bounds__(kThreads) void format8_tiles(const void* __restrict__ xin, void* __restrict__ out, Fmt8 f,
                                                          Mode8 m, uint64_t seed, uint64_t blk0, uint32_t xcd_lg) {
  constexpr int WW = W == 0 ? 1 : W;
  typedef WgTile<WW> T;
  __shared__ uint4 strip[T::BLOCKS];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  if constexpr (SRC == kSrcFP32) {
    const float* x = reinterpret_cast<const float*>(xin);
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x, xcd_lg);
    const uint64_t row0 = (uint64_t)tile * (T::ELEMS / 4) + (uint64_t)(wave * (kWaveElems / 4) + lane);   // units of 4 elements
    f32x4 v[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) v[k] = load_stream4(x + 4 * (row0 + (uint64_t)(k * 64)));
    if constexpr (W != 0) {
      fill_wg_bits<WW>(strip, threadIdx.x, blk0 + (uint64_t)tile * T::BLOCKS, seed, 0);
      __syncthreads();
    }
    uint32_t umax = 0;
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
      umax = max(umax, max(max(__float_as_uint(v[k].x) & 0x7FFFFFFFu, __float_as_uint(v[k].y) & 0x7FFFFFFFu),
                           max(__float_as_uint(v[k].z) & 0x7FFFFFFFu, __float_as_uint(v[k].w) & 0x7FFFFFFFu)));
    }
    const bool checked = __any(umax > 0x7F800000u);   // wave-uniform: a NaN among the wave's elements
    const float grid_scale = W == 32 ? __builtin_amdgcn_ldexpf(f.sub_scale, -(int)m.shift) : 0.0f;
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
      const uint32_t b[4] = {__float_as_uint(v[k].x), __float_as_uint(v[k].y), __float_as_uint(v[k].z),
                             __float_as_uint(v[k].w)};
      uint32_t n4[4] = {0, 0, 0, 0};
      if constexpr (W != 0) row_draws4<WW>(strip, wave, lane, k, m.nbits, n4);
      if constexpr (WIDE) {
        const uint2 c = round4_codes16<TIES>(b, n4, checked, f, m);
        __builtin_nontemporal_store((uint64_t)c.x | ((uint64_t)c.y << 32), reinterpret_cast<uint64_t*>(out) + row0 + (uint64_t)(k * 64));
      } else {
        __builtin_nontemporal_store(round4_bytes<TIES, W == 32>(b, n4, checked, f, m, grid_scale),
                                    reinterpret_cast<uint32_t*>(out) + row0 + (uint64_t)(k * 64));
      }
    }
  } else {
    const uint16_t* x = reinterpret_cast<const uint16_t*>(xin);
    const int e0 = wave * kWaveElems + 8 * lane;                                  // tile-relative first element
    const uint32_t tile = xcd_tile(blockIdx.x, gridDim.x, xcd_lg);
    const uint64_t g0 = (uint64_t)tile * T::ELEMS + (uint64_t)e0;           // call-relative first element
    const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + g0));
    if constexpr (W != 0) {
      fill_wg_bits<WW>(strip, threadIdx.x, blk0 + (uint64_t)tile * T::BLOCKS, seed, 0);
      __syncthreads();
    }
    const uint32_t words[4] = {q.x, q.y, q.z, q.w};
    uint32_t b[8];
    uint32_t umax = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      b[j] = widen16<SRC>((words[j >> 1] >> (16 * (j & 1))) & 0xFFFFu);
      umax = max(umax, b[j] & 0x7FFFFFFFu);
    }
    const bool checked = __any(umax > 0x7F800000u);
    const float grid_scale = W == 32 ? __builtin_amdgcn_ldexpf(f.sub_scale, -(int)m.shift) : 0.0f;
    uint32_t n[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (W != 0) read_wg_bits8<WW>(strip, e0, m.nbits, n);
    const uint32_t b_lo[4] = {b[0], b[1], b[2], b[3]}, b_hi[4] = {b[4], b[5], b[6], b[7]};
    const uint32_t n_lo[4] = {n[0], n[1], n[2], n[3]}, n_hi[4] = {n[4], n[5], n[6], n[7]};
    if constexpr (WIDE) {
      const uint2 lo = round4_codes16<TIES>(b_lo, n_lo, checked, f, m), hi = round4_codes16<TIES>(b_hi, n_hi, checked, f, m);
      u32x4 c;
      c.x = lo.x; c.y = lo.y; c.z = hi.x; c.w = hi.y;
      __builtin_nontemporal_store(c, reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(out) + g0));
    } else {
      const uint32_t lo = round4_bytes<TIES, W == 32>(b_lo, n_lo, checked, f, m, grid_scale);
      const uint32_t hi = round4_bytes<TIES, W == 32>(b_hi, n_hi, checked, f, m, grid_scale);
      __builtin_nontemporal_store((uint64_t)lo | ((uint64_t)hi << 32), reinterpret_cast<uint64_t*>(reinterpret_cast<uint8_t*>(out) + g0));
    }
  }
}

// ------------------------------------------------- 16-bit sources through a table over their magnitudes ---
// A 16-bit source has 2^15 magnitudes, and everything round8 computes before the element's random integer enters
// depends on the magnitude alone.  One workgroup per compute unit tabulates that part once (128 KiB of LDS) and then
// streams tiles through it: per element one table read, the magnitude code (entry + (n << shift)) >> 24, and the
// signs of four bytes at a time.  An entry is round8_fixed_part's sum, which at or below M stays at or below max_code
// under every n; above M, where no random bits apply, it is the finished magnitude code in the top byte over zero
// fraction bits, which the n << shift of any n leaves where it is.  A wave whose tile holds a NaN rounds that tile
// with round8 itself.
//
// Geometry: 1024 threads in four groups of 256; a pass of the loop takes 16 consecutive tiles, group g the tiles
// 4 q + g, q = 0 .. 3, a lane 8 consecutive codes of each (16-byte loads, issued one pass ahead; 8-byte stores).
// Every wave draws the Philox blocks of its own 4 x 512 elements into a strip of its own (64 blocks, one per lane;
// with 8-bit slots in two halves), so the loop has no workgroup barrier.
constexpr int kLutThreads = 1024;
constexpr int kLutPassTiles = 16;
constexpr int kLutEntries = 1 << 15;

template <int SRC, bool TIES>
__device__ __forceinline__ uint32_t lut_entry(uint32_t magnitude16, const Fmt8& f, const Mode8& m) {
  const uint32_t bits = widen16<SRC>(magnitude16);
  if (bits > 0x7F800000u) return f.nan_code << 24;   // a NaN: never read on the table path
  bool above;
  const uint32_t sum = round8_fixed_part<TIES, false>(bits, f, m, &above);
  if (!above) return sum;
  const uint32_t mag = sum >> 24;
  return (mag > f.max_code ? f.over_code : mag) << 24;
}

template <int SRC, int W>
__global__ __launch_bounds__(kLutThreads) void format8_lut_tiles(const uint16_t* __restrict__ x, uint8_t* __restrict__ out, Fmt8 f,
                                                                 Mode8 m, uint64_t seed, uint64_t blk0, uint32_t ntiles) {
  constexpr int WW = W == 0 ? 1 : W;
  constexpr int BLOCKS = WgTile<WW>::BLOCKS;                  // Philox blocks per tile
  constexpr int WAVE_BLOCKS = BLOCKS / kWavesPerBlock;        // ... per wave's 512 elements of a tile: 4 W
  constexpr int Q_PER_DRAW = 64 / WAVE_BLOCKS >= 4 ? 4 : 64 / WAVE_BLOCKS;                    // tiles of a wave one draw covers
  constexpr uint32_t NAN_ABOVE = (SRC == kSrcBF16 ? 0x7F80u : 0x7C00u) << 2;                  // as a byte offset into the table
  static_assert(W == 0 || (Q_PER_DRAW >= 1 && Q_PER_DRAW * WAVE_BLOCKS <= 64), "a draw is at most one block per lane");
  __shared__ uint32_t lut[kLutEntries];
  __shared__ uint4 strips[W == 0 ? 1 : kLutThreads / 64][W == 0 ? 1 : 64];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // 0 .. 15
  const int group = wave >> 2;
  const int e0 = 8 * (tid & 255);                             // tile-relative first element
  {
    // 1024 consecutive magnitudes per step.  A step that lies wholly above M and at or above the clamp (every entry is
    // the one of the clamp itself; NaN entries are never read) or wholly below one unit of the code space (the pattern is 0, plus
    // the sticky bit of a non-zero value) is filled with these constants; most of a bf16 source's range is such.
    const auto entry = [&](uint32_t mag16) { return m.ties ? lut_entry<SRC, true>(mag16, f, m) : lut_entry<SRC, false>(mag16, f, m); };
    const uint32_t at_clamp = entry(SRC == kSrcBF16 ? 0x7F80u : 0x7C00u), at_zero = entry(0u), below_one = entry(1u);
    for (int i0 = 0; i0 < kLutEntries; i0 += kLutThreads) {
      const uint32_t first = widen16<SRC>((uint32_t)i0), last = widen16<SRC>((uint32_t)(i0 + kLutThreads - 1));
      const int i = i0 + tid;
      if (first >= f.u_clamp && first > f.u_max) lut[i] = at_clamp;
      else if (__uint_as_float(last) * f.sub_scale < 1.0f && last < f.u_sub) lut[i] = i == 0 ? at_zero : below_one;
      else lut[i] = entry((uint32_t)i);
    }
  }
  __syncthreads();
  const uint32_t passes = (ntiles + (uint32_t)kLutPassTiles - 1u) / (uint32_t)kLutPassTiles;
  uint4* const strip = strips[W == 0 ? 0 : wave];
  // a tile past the end reads the last one again and stores nothing; the loads of a pass are issued one pass ahead
  const auto load_pass = [&](uint32_t pass, u32x4 (&v)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t tile = min(pass * (uint32_t)kLutPassTiles + (uint32_t)(4 * q + group), ntiles - 1u);
      v[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + (uint64_t)tile * kTileElems + (uint64_t)e0));
    }
  };
  u32x4 ahead[4];
  load_pass(blockIdx.x, ahead);
  for (uint32_t pass = blockIdx.x; pass < passes; pass += gridDim.x) {
    const uint32_t tile0 = pass * (uint32_t)kLutPassTiles;
    u32x4 v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = ahead[q];
    load_pass(min(pass + gridDim.x, passes - 1u), ahead);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if constexpr (W != 0) {
        if (q % Q_PER_DRAW == 0) {   // the blocks of this wave's elements in tiles 4 (q + qq) + group, qq < Q_PER_DRAW
          __builtin_amdgcn_wave_barrier();   // the wave's own LDS traffic keeps program order; this keeps the compiler to it
          if (lane < Q_PER_DRAW * WAVE_BLOCKS) {
            const uint32_t tile = tile0 + (uint32_t)(4 * (q + lane / WAVE_BLOCKS) + group);
            uint32_t o[4];
            philox_block(blk0 + (uint64_t)tile * BLOCKS + (uint64_t)((wave & 3) * WAVE_BLOCKS + lane % WAVE_BLOCKS), seed, 0, o);
            strip[lane] = make_uint4(o[0], o[1], o[2], o[3]);
          }
          __builtin_amdgcn_wave_barrier();
        }
      }
      const uint32_t tile = tile0 + (uint32_t)(4 * q + group);
      const uint32_t words[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
      uint32_t n[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if constexpr (W != 0) read_wg_bits8<WW>(strip + (q % Q_PER_DRAW) * WAVE_BLOCKS, 8 * lane, m.nbits, n);
      uint32_t at[8], at_max = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        at[j] = (j & 1) ? (words[j >> 1] >> 14) & 0x1FFFCu : (words[j >> 1] << 2) & 0x1FFFCu;
        at_max = max(at_max, at[j]);
      }
      uint32_t c[8], lo, hi;
      if (__any(at_max > NAN_ABOVE)) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint32_t bits = widen16<SRC>((words[j >> 1] >> (16 * (j & 1))) & 0xFFFFu);
          c[j] = m.ties ? round8<true, true>(bits, n[j], f, m) : round8<false, true>(bits, n[j], f, m);
        }
        lo = pack4_bytes(c[0], c[1], c[2], c[3]);
        hi = pack4_bytes(c[4], c[5], c[6], c[7]);
      } else {
        // an entry at or below M plus any n << shift stays at or below max_code; one above M is a finished code
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint32_t entry = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(lut) + at[j]);
          c[j] = (entry + (n[j] << m.shift)) >> 24;
        }
        // the top bytes of four 16-bit codes: bytes 1 and 3 of each of two words
        lo = with_signs4(pack4_bytes(c[0], c[1], c[2], c[3]), __builtin_amdgcn_perm(words[1], words[0], 0x07050301u), f);
        hi = with_signs4(pack4_bytes(c[4], c[5], c[6], c[7]), __builtin_amdgcn_perm(words[3], words[2], 0x07050301u), f);
      }
      if (tile < ntiles) {
        __builtin_nontemporal_store((uint64_t)lo | ((uint64_t)hi << 32),
                                    reinterpret_cast<uint64_t*>(out + (uint64_t)tile * kTileElems + (uint64_t)e0));
      }
    }
  }
}

// One thread per element: any alignment, any offset, ragged heads and tails.  W = 0: no bits.
template <int SRC, bool TIES, bool WIDE>
__global__ __launch_bounds__(kThreads) void format8_elems(const void* __restrict__ xin, void* __restrict__ out, uint64_t n,
                                                          Fmt8 f, Mode8 m, int W, int log2_per_block, uint64_t seed,
                                                          uint64_t offset) {
  const uint64_t j = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (j >= n) return;
  uint32_t bits;
  if constexpr (SRC == kSrcFP32) bits = __float_as_uint(reinterpret_cast<const float*>(xin)[j]);
  else bits = widen16<SRC>(reinterpret_cast<const uint16_t*>(xin)[j]);
  uint32_t rnd = 0;
  if (W != 0) rnd = element_bits(offset + j, log2_per_block, W, m.nbits, seed, 0);
  if constexpr (WIDE) {   // at most 16 random bits here
    reinterpret_cast<uint16_t*>(out)[j] = (uint16_t)round8<TIES, true, true>(bits, rnd, f, m);
  } else {
    reinterpret_cast<uint8_t*>(out)[j] =
        (uint8_t)(m.nbits > (uint32_t)kMaxTileNbits ? round8_wide(bits, rnd, f, m) : round8<TIES, true>(bits, rnd, f, m));
  }
}

namespace {

template <int SRC, bool TIES, bool WIDE>
hipError_t launch_tiles_w(int W, const void* x, void* out, uint64_t ntiles, const Fmt8& f, const Mode8& m, uint64_t seed,
                          uint64_t blk0, hipStream_t stream) {
  const dim3 grid((unsigned)ntiles), block(kThreads);
#define FBSR_F8_LAUNCH(WW) hipLaunchKernelGGL((format8_tiles<SRC, TIES, WW, WIDE>), grid, block, 0, stream, x, out, f, m, seed, blk0, kXcdLgFormat8)
  switch (W) {
    case 0: FBSR_F8_LAUNCH(0); break;
    case 1: FBSR_F8_LAUNCH(1); break;
    case 2: FBSR_F8_LAUNCH(2); break;
    case 4: FBSR_F8_LAUNCH(4); break;
    case 8: FBSR_F8_LAUNCH(8); break;
    case 16: FBSR_F8_LAUNCH(16); break;
    default:
      if constexpr (WIDE) return hipErrorInvalidValue;   // 16-bit codes take at most 16 random bits (checked by the caller)
      else FBSR_F8_LAUNCH(32);
      break;
  }
#undef FBSR_F8_LAUNCH
  return hipGetLastError();
}

// The table kernel pays for its table (2^15 entries per workgroup) from 2^26 elements on; it needs the
// device to grant a workgroup its 144 KiB of LDS and at most 8 random bits.
constexpr uint64_t kLutMinTiles = (uint64_t)1 << 15;

struct LutDevice {
  int checked = 0, units = 0, lds = 0;
};

inline bool lut_device(int* units) {
  static LutDevice known[64];
  static std::mutex guard;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
  std::lock_guard<std::mutex> lock(guard);
  LutDevice& d = known[dev];
  if (!d.checked) {
    if (hipDeviceGetAttribute(&d.units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) d.units = 0;
    if (hipDeviceGetAttribute(&d.lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) d.lds = 0;
    d.checked = 1;
  }
  *units = d.units;
  return d.units > 0 && d.lds >= (int)(kLutEntries * 4 + kLutThreads * 16);
}

template <int SRC>
hipError_t launch_lut_tiles(int W, const uint16_t* x, uint8_t* out, uint64_t ntiles, const Fmt8& f, const Mode8& m, uint64_t seed,
                            uint64_t blk0, int units, hipStream_t stream) {
  const uint64_t passes = (ntiles + kLutPassTiles - 1) / kLutPassTiles;
  const dim3 grid((unsigned)(passes < (uint64_t)units ? passes : (uint64_t)units)), block(kLutThreads);
#define FBSR_LUT_LAUNCH(WW) hipLaunchKernelGGL((format8_lut_tiles<SRC, WW>), grid, block, 0, stream, x, out, f, m, seed, blk0, (uint32_t)ntiles)
  switch (W) {
    case 0: FBSR_LUT_LAUNCH(0); break;
    case 1: FBSR_LUT_LAUNCH(1); break;
    case 2: FBSR_LUT_LAUNCH(2); break;
    case 4: FBSR_LUT_LAUNCH(4); break;
    default: FBSR_LUT_LAUNCH(8); break;
  }
#undef FBSR_LUT_LAUNCH
  return hipGetLastError();
}

template <int SRC, bool TIES, bool WIDE>
hipError_t run(const void* xin, void* outv, uint64_t n, const Fmt8& f, const Mode8& m, uint64_t seed, uint64_t offset,
               hipStream_t stream) {
  constexpr uint64_t isize = SRC == kSrcFP32 ? 4 : 2;
  constexpr uint64_t osize = WIDE ? 2 : 1;
  constexpr uint64_t oalign = (SRC == kSrcFP32 ? 4 : 8) * osize;
  const char* x = reinterpret_cast<const char*>(xin);
  char* out = reinterpret_cast<char*>(outv);
  const int W = m.nbits ? slot_width((int)m.nbits) : 0;
  Split s = split_range(n, offset, W ? W : 8, W == 0, reinterpret_cast<uintptr_t>(x), isize, 16,
                        reinterpret_cast<uintptr_t>(out), osize, oalign);
  return run_split(
      s, n,
      [&](uint64_t first, uint64_t count) {
        hipLaunchKernelGGL((format8_elems<SRC, TIES, WIDE>), elems_grid(count), dim3(kThreads), 0, stream,
                           reinterpret_cast<const void*>(x + first * isize), reinterpret_cast<void*>(out + first * osize), count, f, m,
                           W, W ? log2_of(128 / W) : 0, seed, offset + first);
        return hipGetLastError();
      },
      [&](uint64_t first, uint64_t count) {
        const uint64_t blk0 = W ? (offset + first) / (uint64_t)(128 / W) : 0;
        if constexpr (SRC != kSrcFP32 && !WIDE) {
          int units = 0;
          if (count >= kLutMinTiles && W <= 8 && lut_device(&units)) {
            return launch_lut_tiles<SRC>(W, reinterpret_cast<const uint16_t*>(x + first * isize),
                                         reinterpret_cast<uint8_t*>(out + first * osize), count, f, m, seed, blk0, units, stream);
          }
        }
        return launch_tiles_w<SRC, TIES, WIDE>(W, x + first * isize, out + first * osize, count, f, m, seed, blk0, stream);
      });
}

template <int SRC, bool WIDE>
hipError_t run_t(const void* x, void* out, uint64_t n, const Fmt8& f, const Mode8& m, uint64_t seed, uint64_t offset,
                 hipStream_t stream) {
  if (m.ties) return run<SRC, true, WIDE>(x, out, n, f, m, seed, offset, stream);
  return run<SRC, false, WIDE>(x, out, n, f, m, seed, offset, stream);
}

template <bool WIDE>
hipError_t run_s(const void* x, int src, void* out, uint64_t n, const Fmt8& f, const Mode8& m, uint64_t seed, uint64_t offset,
                 hipStream_t stream) {
  switch (src) {
    case kSrcBF16: return run_t<kSrcBF16, WIDE>(x, out, n, f, m, seed, offset, stream);
    case kSrcFP16: return run_t<kSrcFP16, WIDE>(x, out, n, f, m, seed, offset, stream);
    default: return run_t<kSrcFP32, WIDE>(x, out, n, f, m, seed, offset, stream);
  }
}

}  // namespace

hipError_t launch_round_format8(const void* x, int src, uint8_t* out, uint64_t n, const Fmt8& f, const Mode8& m,
                                uint64_t seed, uint64_t offset, hipStream_t stream) {
  return run_s<false>(x, src, out, n, f, m, seed, offset, stream);
}

hipError_t launch_round_format16(const void* x, int src, uint16_t* out, uint64_t n, const Fmt8& f, const Mode8& m,
                                 uint64_t seed, uint64_t offset, hipStream_t stream) {
  return run_s<true>(x, src, out, n, f, m, seed, offset, stream);
}

}  // namespace fbsr
