// fbsr_stats_common.h -- device helpers shared by the two statistics kernels (fixed formats: fbsr_stats.hip; formats
// given by a descriptor: fbsr_stats8.hip).
#pragma once
#include <type_traits>

#include "fbsr_device.h"

namespace fbsr {

// End of a bin in global indices, saturating (group may be as large as 2^62, so (bin + 1) * group can pass 2^64).
__device__ __forceinline__ uint64_t bin_end(uint64_t bin, uint64_t group) {
  const uint64_t k = bin + 1;
  return __umul64hi(k, group) != 0 ? ~(uint64_t)0 : k * group;
}

// Sum over the wave in a fixed tree: quads, eights and sixteens by DPP, the rows of 16 by two exchanges through LDS
// hardware.  Every lane ends with the same bits.
__device__ __forceinline__ double wave_total(double v) {
  auto dpp = [](double a, auto ctrl) {
    constexpr int C = decltype(ctrl)::value;
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(a), C, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(a), C, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
  };
  v += dpp(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
  v += dpp(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
  v += dpp(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
  v += dpp(v, std::integral_constant<int, 0x140>{});   // row_mirror
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

// The 4 W random bits of four consecutive elements whose first has index e0 (a multiple of 4) in the bit string
// `strip` holds (element e at bit e W), right-aligned in a 64-bit word.
template <int W>
__device__ __forceinline__ uint64_t read_row_bits(const uint4* strip, int e0) {
  const unsigned char* base = reinterpret_cast<const unsigned char*>(strip);
  if constexpr (W == 16) {
    return *reinterpret_cast<const uint64_t*>(base + e0 * 2);
  } else if constexpr (W == 8) {
    return *reinterpret_cast<const uint32_t*>(base + e0);
  } else if constexpr (W == 4) {
    return *reinterpret_cast<const uint16_t*>(base + e0 / 2);
  } else if constexpr (W == 2) {
    return base[e0 / 4];
  } else {
    return (uint32_t)(base[e0 / 8] >> (e0 & 4)) & 0xFu;
  }
}

}  // namespace fbsr
