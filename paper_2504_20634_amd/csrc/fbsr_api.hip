// fbsr_api.hip -- the C ABI declared in include/fbsr.h: host-side argument checking and
// dispatch.  Every check happens before anything is enqueued.
#include "../../include/fbsr.h"
#include "fbsr_launch.h"

namespace {

bool valid_fmt(int fmt) { return fmt == FBSR_FMT_BF16 || fmt == FBSR_FMT_E4M3 || fmt == FBSR_FMT_E5M2; }

int check_common(int variant, int nbits, uint64_t n, uint64_t offset) {
  if (variant < FBSR_RNE || variant > FBSR_SRC) return FBSR_EINVAL;
  if (variant != FBSR_RNE && (nbits < 1 || nbits > FBSR_MAX_NBITS)) return FBSR_EINVAL;
  if (n > fbsr::kMaxElems || offset > UINT64_MAX - n) return FBSR_EINVAL;
  return FBSR_OK;
}

bool misaligned(const void* p, uintptr_t a) { return reinterpret_cast<uintptr_t>(p) % a != 0; }

uint64_t code_bytes(int fmt) { return fmt == FBSR_FMT_BF16 ? 2 : 1; }

}  // namespace

extern "C" {

int fbsr_round(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
               uint64_t offset, void* stream) {
  if (!valid_fmt(fmt)) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset);
  if (c != FBSR_OK) return c;
  if (n == 0) return FBSR_OK;
  if (x == nullptr || out == nullptr) return FBSR_EINVAL;
  if (misaligned(x, 4) || misaligned(out, code_bytes(fmt))) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_round(x, out, n, fmt, variant, nbits, seed, offset,
                                          reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_round_from16(const void* x, void* out, uint64_t n, int src_fmt, int fmt, int variant, int nbits,
                      uint64_t seed, uint64_t offset, void* stream) {
  if (fmt != FBSR_FMT_E4M3 && fmt != FBSR_FMT_E5M2) return FBSR_EINVAL;
  if (src_fmt != FBSR_SRC_BF16 && src_fmt != FBSR_SRC_FP16) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset);
  if (c != FBSR_OK) return c;
  if (n == 0) return FBSR_OK;
  if (x == nullptr || out == nullptr) return FBSR_EINVAL;
  if (misaligned(x, 2)) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_round_from16(x, out, n, src_fmt, fmt, variant, nbits, seed, offset,
                                                 reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_sgd_update(void* w, const float* g, uint64_t n, float lr, int variant, int nbits, uint64_t seed,
                    uint64_t step, uint64_t offset, void* stream) {
  const int c = check_common(variant, nbits, n, offset);
  if (c != FBSR_OK) return c;
  if (n == 0) return FBSR_OK;
  if (w == nullptr || g == nullptr) return FBSR_EINVAL;
  if (misaligned(g, 4) || misaligned(w, 2)) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_sgd(w, g, n, lr, variant, nbits, seed, step, offset,
                                        reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_round_block_scaled(const float* x, void* out, void* scales, uint64_t n, int fmt, int variant, int nbits,
                            uint64_t seed, uint64_t offset, void* stream) {
  if (fmt != FBSR_FMT_E4M3 && fmt != FBSR_FMT_E5M2) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset);
  if (c != FBSR_OK) return c;
  if (n == 0) return FBSR_OK;
  if (x == nullptr || out == nullptr || scales == nullptr) return FBSR_EINVAL;
  if (misaligned(x, 4)) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_round_block_scaled(x, reinterpret_cast<uint8_t*>(out), reinterpret_cast<uint8_t*>(scales),
                                                       n, fmt, variant, nbits, seed, offset,
                                                       reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_qat_adamw_step(void* w8, const void* g16, void* m16, void* v16, uint64_t n, int fmt, const fbsr_adamw* p,
                        int variant, int nbits, uint64_t seed, uint64_t step, uint64_t offset, void* stream) {
  if (fmt != FBSR_FMT_E4M3 && fmt != FBSR_FMT_E5M2) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset);
  if (c != FBSR_OK) return c;
  if (p == nullptr) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (w8 == nullptr || g16 == nullptr || m16 == nullptr || v16 == nullptr) return FBSR_EINVAL;
  if (misaligned(g16, 2) || misaligned(m16, 2) || misaligned(v16, 2)) return FBSR_EALIGN;
  const fbsr::AdamWScalars sc = {p->lr, p->beta1, p->beta2, p->eps, p->weight_decay, p->bias_corr1, p->bias_corr2};
  const hipError_t e = fbsr::launch_qat_adamw(reinterpret_cast<uint8_t*>(w8), reinterpret_cast<const uint16_t*>(g16),
                                              reinterpret_cast<uint16_t*>(m16), reinterpret_cast<uint16_t*>(v16), n, fmt,
                                              sc, variant, nbits, seed, step, offset,
                                              reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

uint64_t fbsr_bias_stats_workspace_bytes(uint64_t n, uint32_t nbins) {
  (void)nbins;
  // one record per (chunk, bin it touches), sized for the smallest group the chunked kernel takes
  const uint64_t chunk = (uint64_t)fbsr::kStatsChunkTiles * fbsr::kTileElems;
  return (n / chunk + 1) * fbsr::kStatsMaxSlots * fbsr::kStatsRecordDoubles * sizeof(double);
}

int fbsr_bias_stats(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
                    uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins, double* stats,
                    void* workspace, uint64_t workspace_bytes, void* stream) {
  if (!valid_fmt(fmt)) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset);
  if (c != FBSR_OK) return c;
  if (group == 0 || group > ((uint64_t)1 << 62)) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (x == nullptr || stats == nullptr || workspace == nullptr) return FBSR_EINVAL;
  if (misaligned(x, 4) || misaligned(stats, 8) || misaligned(workspace, 8)) return FBSR_EALIGN;
  if (out != nullptr && misaligned(out, code_bytes(fmt))) return FBSR_EALIGN;
  const uint64_t bin_lo = offset / group, bin_hi = (offset + n - 1) / group;
  if (bin_lo < first_bin || bin_hi - first_bin >= nbins) return FBSR_ERANGE;
  if (workspace_bytes < fbsr_bias_stats_workspace_bytes(n, nbins)) return FBSR_ERANGE;
  const hipError_t e =
      fbsr::launch_stats(x, out, n, fmt, variant, nbits, seed, offset, group, first_bin, nbins, stats,
                         reinterpret_cast<double*>(workspace), reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

const char* fbsr_strerror(int status) {
  switch (status) {
    case FBSR_OK: return "ok";
    case FBSR_EINVAL: return "invalid argument";
    case FBSR_EALIGN: return "pointer not aligned to its element type";
    case FBSR_ERANGE: return "element outside the bins, or workspace too small";
    case FBSR_EDEVICE: return "HIP runtime error at launch";
  }
  return "unknown status";
}

int fbsr_version(void) { return 100; }

}  // extern "C"
