// Host-only stand-ins for the kernel launchers, so that the C ABI's argument checks (csrc/fbsr_api.hip) can be
// linked and run under the host sanitizers without any device code.  Every stand-in reports success and launches
// nothing; tests/test_sanitizers.py builds this file together with fbsr_api.hip.
#include "../paper_2504_20634_amd/csrc/fbsr_launch.h"

namespace fbsr {

hipError_t launch_round(const float*, void*, uint64_t, int, int, int, uint64_t, uint64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_stream41(const float*, uint8_t*, uint64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_check_division(const float*, const float*, uint64_t, unsigned long long*, hipStream_t) { return hipSuccess; }
hipError_t launch_check_corrected_root(const AdamWScalars&, unsigned long long*, hipStream_t) { return hipSuccess; }
hipError_t launch_stream75(uint8_t*, const uint16_t*, uint16_t*, uint16_t*, uint64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_round_from16(const void*, void*, uint64_t, int, int, int, int, uint64_t, uint64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_sgd(void*, const float*, uint64_t, float, int, int, uint64_t, uint64_t, uint64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_round_block_scaled(const float*, uint8_t*, uint8_t*, uint64_t, int, int, int, uint64_t, uint64_t, hipStream_t) {
  return hipSuccess;
}
hipError_t launch_qat_adamw_format8(uint8_t*, const uint16_t*, uint16_t*, uint16_t*, uint64_t, const Fmt8&, const Mode8&,
                                    const Table8&, const AdamWScalars&, uint64_t, uint64_t, uint64_t, hipStream_t) {
  return hipSuccess;
}
hipError_t launch_qat_adamw(uint8_t*, const uint16_t*, uint16_t*, uint16_t*, uint64_t, int, const AdamWScalars&, int, int,
                            uint64_t, uint64_t, uint64_t, hipStream_t) {
  return hipSuccess;
}
hipError_t launch_round_format8(const void*, int, uint8_t*, uint64_t, const Fmt8&, const Mode8&, uint64_t, uint64_t, hipStream_t) {
  return hipSuccess;
}
hipError_t launch_round_format16(const void*, int, uint16_t*, uint64_t, const Fmt8&, const Mode8&, uint64_t, uint64_t, hipStream_t) {
  return hipSuccess;
}
hipError_t launch_stats(const float*, void*, uint64_t, int, int, int, uint64_t, uint64_t, uint64_t, uint64_t, uint32_t, double*,
                        double*, hipStream_t) {
  return hipSuccess;
}
hipError_t launch_stats_format8(const float*, uint8_t*, uint64_t, const Fmt8&, const Mode8&, const Table8&, int, int, uint64_t,
                                uint64_t, uint64_t, uint64_t, double*, double*, hipStream_t) {
  return hipSuccess;
}
hipError_t static_scratch(double** ptr) {
  static double none[1];
  *ptr = none;
  return hipSuccess;
}

}  // namespace fbsr
