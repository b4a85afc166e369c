// fbsr_launch.h -- host-side planning shared by the kernel translation units and the C ABI.
#pragma once

#include "fbsr_device.h"

namespace fbsr {

// Slot width: the smallest power of two >= nbits.
inline int slot_width(int nbits) {
  int w = 1;
  while (w < nbits) w *= 2;
  return w;
}

inline int log2_of(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

// How a call over [0, n) is cut: `head` elements for the per-element kernel (up to the first
// global index that starts a Philox block), `ntiles` whole tiles for the vector kernel, and
// the rest for the per-element kernel again.  The vector kernel is used only when both
// buffers are suitably aligned at the first tile.
struct Split {
  uint64_t head;
  uint64_t ntiles;
  uint64_t tile_elems;
};

// in_addr / out_addr: addresses of element 0; *_esize: bytes per element; *_align: alignment
// the vector kernel needs at a tile start.  out_addr may be 0 (no output buffer).
inline Split split_range(uint64_t n, uint64_t offset, int W, bool no_bits, uintptr_t in_addr, uint64_t in_esize,
                         uint64_t in_align, uintptr_t out_addr, uint64_t out_esize, uint64_t out_align,
                         uintptr_t in2_addr = 0, uint64_t in2_esize = 0, uint64_t in2_align = 1,
                         uint64_t tile_elems = (uint64_t)kTileElems) {
  Split s;
  s.tile_elems = tile_elems;   // one workgroup tile, unless the kernel works in other units
  const uint64_t per_block = no_bits ? 1 : (uint64_t)(128 / W);
  uint64_t head = (per_block - offset % per_block) % per_block;
  if (head > n) head = n;
  s.head = head;
  s.ntiles = (n - head) / s.tile_elems;
  const bool aligned = (in_addr + head * in_esize) % in_align == 0 &&
                       (out_addr == 0 || (out_addr + head * out_esize) % out_align == 0) &&
                       (in2_addr == 0 || (in2_addr + head * in2_esize) % in2_align == 0);
  if (!aligned || s.ntiles == 0) {
    s.head = 0;   // everything goes through the per-element kernel in one piece
    s.ntiles = 0;
  }
  return s;
}

// Largest element count one per-element launch may cover (keeps the total thread count of a launch
// far below 2^32).
constexpr uint64_t kMaxElemsPerLaunch = (uint64_t)1 << 30;
// Largest tile count one tile-kernel launch may cover (2^30 threads per launch).
constexpr uint64_t kMaxTilesPerLaunch = (uint64_t)1 << 22;
// log2 of the run of consecutive tiles (for the narrow-source kernel: pairs of tiles) an XCD takes within a launch
// (xcd_tile), per kernel family; 0 keeps the identity order.  From sweeps over 0..12 on 2^28 elements: the kernels that
// read fp32 gain 4-5 % at runs of 128-256 tiles (fp32 -> fp8 6.25 -> 6.57 TB/s, fp32 -> bf16 6.40 -> 6.70, the SGD
// update 6.15 -> 6.38), a plain 16-bit -> 8-bit stream with 4096 elements per workgroup 5 % at runs of 128 (6.35 ->
// 6.65), the QAT step's 7 : 5 in-place stream 3 % at runs of 128 (its no-arithmetic probe 5.64 -> 5.83); for the
// block-scaled and the generic-format kernels no run length differs from the identity by more than run-to-run noise.
constexpr uint32_t kXcdLgRound = 7, kXcdLgRoundBf16 = 8, kXcdLgSgd = 7, kXcdLgRound16 = 7, kXcdLgBlock = 0, kXcdLgFormat8 = 0, kXcdLgQat = 7;
// The fp32 -> 8-bit rounding kernels (and their no-arithmetic probe) take workgroups of 8 waves, 4096 elements: at
// sustained clocks 84.2 % of the HBM peak against 82.8 % with 4 waves and 75 % with 16 (runs of 128 such tiles per XCD;
// 83.8 % with 256, 83.1 % with 64).  fp32 -> bf16 (6 bytes per element) loses 1 % that way and keeps 4 waves.
constexpr int kRoundWaves = 8;
constexpr int kRoundThreads = 64 * kRoundWaves;
constexpr int kRoundTileElems = kRoundWaves * kWaveElems;
template <int FMT> struct RoundGeometry {
  static constexpr int WAVES = Fx<FMT>::kIsFp8 ? kRoundWaves : kWavesPerBlock;
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int TILE_ELEMS = WAVES * kWaveElems;
  static constexpr uint32_t XCD_LG = Fx<FMT>::kIsFp8 ? kXcdLgRound : kXcdLgRoundBf16;
};
// Up to 16 random bits per element use slots of at most 16 bits and a code space with 24 fraction bits.  With more (the
// rounding entry points take up to 24) every tile kernel has a flavour with 32-bit slots: the fp8 targets through the
// hardware converts where those are exact and otherwise, like bf16 and the generic formats, in the same code space with
// the target-subnormal positions taken from an exact float product (round_pattern_many); the per-element kernels keep
// 32 fraction bits and a sticky bit (round_pattern_wide).
constexpr int kMaxTileNbits = 16;
// Largest n the library accepts.
constexpr uint64_t kMaxElems = (uint64_t)1 << 38;

// Calls launch(first, count) over [0, n) in pieces of at most `piece`; stops at the first error.
template <class Launch>
hipError_t in_pieces(uint64_t n, uint64_t piece, Launch launch) {
  for (uint64_t at = 0; at < n; at += piece) {
    const uint64_t m = n - at < piece ? n - at : piece;
    const hipError_t e = launch(at, m);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Carries out the cut of split_range: elems(first, count) launches the per-element kernel over the
// elements [first, first + count) of the call, tiles(first, count) the tile kernel over `count` whole
// tiles of which the first starts at element `first`.
template <class Elems, class Tiles>
hipError_t run_split(const Split& s, uint64_t n, Elems elems, Tiles tiles) {
  hipError_t e = in_pieces(s.head, kMaxElemsPerLaunch, elems);
  if (e != hipSuccess) return e;
  e = in_pieces(s.ntiles, kMaxTilesPerLaunch,
                [&](uint64_t t0, uint64_t count) { return tiles(s.head + t0 * s.tile_elems, count); });
  if (e != hipSuccess) return e;
  const uint64_t done = s.head + s.ntiles * s.tile_elems;
  return in_pieces(n - done, kMaxElemsPerLaunch, [&](uint64_t at, uint64_t count) { return elems(done + at, count); });
}

inline dim3 elems_grid(uint64_t count) { return dim3((unsigned)((count + kThreads - 1) / kThreads)); }

hipError_t launch_round(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
                        uint64_t offset, hipStream_t stream);

hipError_t launch_stream41(const float* x, uint8_t* out, uint64_t ntiles, hipStream_t stream);
hipError_t launch_stream75(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t ntiles, hipStream_t stream);

hipError_t launch_round_from16(const void* x, void* out, uint64_t n, int src_fmt, int fmt, int variant, int nbits,
                               uint64_t seed, uint64_t offset, hipStream_t stream);

hipError_t launch_sgd(void* w, const float* g, uint64_t n, float lr, int variant, int nbits, uint64_t seed,
                      uint64_t step, uint64_t offset, hipStream_t stream);

hipError_t launch_round_block_scaled(const float* x, uint8_t* out, uint8_t* scales, uint64_t n, int fmt, int variant,
                                    int nbits, uint64_t seed, uint64_t offset, hipStream_t stream);

struct AdamWScalars {
  float lr, beta1, beta2, eps, weight_decay, bias_corr1, bias_corr2;
  // 1 / bias_corr (correctly rounded, computed on the host) and whether the tile kernel may take its shortened
  // divisions and the tabulated square root (both corrections in [2^-20, 1], eps in [2^-28, 2^30]); the caller's
  // struct ends at bias_corr2.
  float rcp_corr1, rcp_corr2;
  int fast_div;
};

// Fills the derived fields of AdamWScalars.
inline void derive_adamw(AdamWScalars* p) {
  const float lo = 0x1p-20f;
  p->fast_div = p->bias_corr1 >= lo && p->bias_corr1 <= 1.0f && p->bias_corr2 >= lo && p->bias_corr2 <= 1.0f &&
                p->eps >= 0x1p-28f && p->eps <= 0x1p30f;
  p->rcp_corr1 = p->fast_div ? 1.0f / p->bias_corr1 : 0.0f;
  p->rcp_corr2 = p->fast_div ? 1.0f / p->bias_corr2 : 0.0f;
}

hipError_t launch_qat_adamw_format8(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t n,
                                    const Fmt8& f, const Mode8& m, const Table8& t, const AdamWScalars& p, uint64_t seed,
                                    uint64_t step, uint64_t offset, hipStream_t stream);

// Device self-checks of the fused step's short arithmetic (fbsr_measure.h).
hipError_t launch_check_division(const float* num, const float* den, uint64_t count, unsigned long long* counts, hipStream_t stream);
hipError_t launch_check_corrected_root(const AdamWScalars& p, unsigned long long* counts, hipStream_t stream);

hipError_t launch_qat_adamw(uint8_t* w8, const uint16_t* g16, uint16_t* m16, uint16_t* v16, uint64_t n, int fmt,
                            const AdamWScalars& p, int variant, int nbits, uint64_t seed, uint64_t step,
                            uint64_t offset, hipStream_t stream);

hipError_t launch_round_format8(const void* x, int src, uint8_t* out, uint64_t n, const Fmt8& f, const Mode8& m,
                                uint64_t seed, uint64_t offset, hipStream_t stream);

hipError_t launch_round_format16(const void* x, int src, uint16_t* out, uint64_t n, const Fmt8& f, const Mode8& m,
                                 uint64_t seed, uint64_t offset, hipStream_t stream);

// Geometry of the statistics kernel: a workgroup takes a chunk of kStatsChunkElems consecutive elements, each of
// its waves a span of kStatsSpanElems of them, walked in pairs of rows (kStatsPairElems = 512 elements: eight per
// lane).  Bins must hold at least kStatsMinGroup elements on this path, so a chunk touches at most
// kStatsMaxBinsPerChunk of them; the first and the last of those may continue in the neighbouring chunks and leave
// one record {sum y, sum e, sum e^2} each in the workspace.
constexpr int kStatsPairElems = kRows * 256;
constexpr int kStatsSpanPairs = 8;
constexpr int kStatsSpanElems = kStatsSpanPairs * kStatsPairElems;
constexpr int kStatsChunkElems = kWavesPerBlock * kStatsSpanElems;
constexpr uint64_t kStatsMinGroup = 512;
constexpr int kStatsMaxBinsPerChunk = kStatsChunkElems / (int)kStatsMinGroup + 2;
constexpr uint64_t kStatsRecordDoubles = 3;
inline uint64_t stats_workspace_bytes(uint64_t n) {
  return (n / (uint64_t)kStatsChunkElems + 2) * 2 * kStatsRecordDoubles * sizeof(double);
}

// fbsr_bias_stats_static: bytes of the workspace array that lives in the library's device image, and the largest
// call it serves (its records need 48 bytes per 16384 elements: 768 KiB at 2^28).
constexpr uint64_t kStaticScratchBytes = (uint64_t)1 << 20;
constexpr uint64_t kStaticMaxElems = (uint64_t)1 << 28;

// Address of that array on the current device (looked up once per device).
hipError_t static_scratch(double** ptr);

// Adds the workspace records of the chunks that cover global indices [i0, i_end) to the caller's statistics (the
// kernel that closes both statistics paths).
hipError_t launch_stats_finalize(const double* records, uint64_t i0, uint64_t i_end, uint64_t group, uint64_t first_bin,
                                 double* stats, hipStream_t stream);

// The statistics for a format given by its descriptor; P and B are the descriptor's (for ulp_t).
hipError_t launch_stats_format8(const float* x, uint8_t* out, uint64_t n, const Fmt8& f, const Mode8& m, const Table8& t,
                                int P, int B, uint64_t seed, uint64_t offset, uint64_t group, uint64_t first_bin,
                                double* stats, double* workspace, hipStream_t stream);

hipError_t launch_stats(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
                        uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins, double* stats,
                        double* workspace, hipStream_t stream);

}  // namespace fbsr
