// fbsr_api.hip -- the C ABI declared in include/fbsr.h: host-side argument checking and
// dispatch.  Every check happens before anything is enqueued.
#include <math.h>
#include <string.h>

#include "../../include/fbsr.h"
#include "../../include/fbsr_measure.h"
#include "fbsr_launch.h"

namespace {

bool valid_fmt(int fmt) { return fmt >= FBSR_FMT_BF16 && fmt <= FBSR_FMT_BINARY8P4; }

bool is_8bit_fmt(int fmt) { return fmt == FBSR_FMT_E4M3 || fmt == FBSR_FMT_E5M2 || fmt == FBSR_FMT_BINARY8P4; }

int check_common(int variant, int nbits, uint64_t n, uint64_t offset, int max_nbits = FBSR_MAX_NBITS) {
  if (variant < FBSR_RNE || variant > FBSR_SRC) return FBSR_EINVAL;
  if (variant != FBSR_RNE && (nbits < 1 || nbits > max_nbits)) return FBSR_EINVAL;
  if (n > fbsr::kMaxElems || offset > UINT64_MAX - n) return FBSR_EINVAL;
  return FBSR_OK;
}

bool misaligned(const void* p, uintptr_t a) { return reinterpret_cast<uintptr_t>(p) % a != 0; }

uint64_t code_bytes(int fmt) { return fmt == FBSR_FMT_BF16 ? 2 : 1; }

// Checks a generic-format descriptor and reduces it to the constants of the code-space arithmetic.
// max_width 8: codes are bytes and the code space has 24 fraction bits.  max_width 16: codes are 16-bit words and the
// code space has 32 - K fraction bits, which must hold every bit an fp32 value drops (24 - P), so P >= K - 8.
bool derive_format8(const fbsr_format8& d, fbsr::Fmt8* f, int max_width = 8) {
  const int K = d.width, P = d.precision, B = d.bias;
  if (K < 2 || K > max_width || P < 1 || P >= K || B < 0 || B > (max_width > 8 ? 127 : 96)) return false;
  const int frac = max_width > 8 ? 32 - K : 24;
  if (frac < 24 - P) return false;
  const int sign_bit = 1 << (K - 1), mag_top = sign_bit - 1;
  if (d.max_code > mag_top || d.max_code < (1 << (P - 1))) return false;   // M must be a normal value
  const bool has_inf = d.inf_code != -1;
  if (has_inf && (d.inf_code <= d.max_code || d.inf_code > mag_top)) return false;
  const bool has_nan = d.nan_code != -1;
  if (has_nan) {
    if (d.nan_code < 0 || d.nan_code > 2 * mag_top + 1) return false;
    const int mag = d.nan_code & mag_top;
    const bool negative = (d.nan_code & sign_bit) != 0;
    const bool spare_magnitude = mag > d.max_code && !(has_inf && mag == d.inf_code);
    const bool minus_zero_code = mag == 0 && negative && d.neg_zero == 0 && d.nan_signed == 0;
    if (!spare_magnitude && !minus_zero_code) return false;
    if (d.nan_signed != 0 && negative) return false;
  }
  const int e_max = d.max_code >> (P - 1), t_max = d.max_code & ((1 << (P - 1)) - 1);
  if (e_max - B > 126) return false;   // M + ulp(M) has to be a finite fp32 value
  const uint32_t ulp = 1u << (24 - P);   // one target ulp of a normal value, in fp32 pattern units
  f->frac = (uint32_t)frac;
  f->shift_p = (uint32_t)(frac - (24 - P));
  f->sub_exp = frac - 2 + B + P;
  f->rebias = (uint32_t)(127 - B) << 23;
  f->u_max = ((uint32_t)(e_max + 127 - B) << 23) | ((uint32_t)t_max * ulp);
  f->u_clamp = has_inf ? f->u_max + 3u * (ulp >> 2) : f->u_max;
  f->u_sub = (uint32_t)(128 - B) << 23;
  f->sub_scale = frac == 24 ? ldexpf(1.0f, 22 + B + P) : 0.0f;   // the 16-bit path scales by sub_exp instead
  const uint32_t m_odd = P == 1 ? 1u : (uint32_t)(d.max_code & 1);   // parity of M's significand
  f->det_add = (1u << (frac - 1)) - 1u + m_odd;
  f->max_code = (uint32_t)d.max_code;
  f->over_code = (uint32_t)(has_inf ? d.inf_code : d.max_code);
  f->remap_over = has_inf && d.inf_code != d.max_code + 1 ? 1u : 0u;
  f->nan_code = (uint32_t)(has_nan ? d.nan_code : d.max_code);
  f->nan_sign = (!has_nan || d.nan_signed != 0) ? (uint32_t)sign_bit : 0u;
  f->sign_bit = (uint32_t)sign_bit;
  f->sign_shift = (uint32_t)(32 - K);
  f->sign_carry = d.neg_zero != 0 ? (uint32_t)sign_bit : (uint32_t)sign_bit - 1u;
  f->unit_lsb = P == 1 ? (1u << frac) : 0u;
  return true;
}

// Value of every byte taken as a code of the (checked) format: Eq. (1), with the descriptor's specials.
void decode_table8(const fbsr_format8& d, fbsr::Table8* t) {
  const int K = d.width, P = d.precision, B = d.bias;
  const int sign_bit = 1 << (K - 1), mag_top = sign_bit - 1;
  for (int byte = 0; byte < 256; ++byte) {
    const int code = byte & (2 * mag_top + 1);   // bits above K are ignored
    const int mag = code & mag_top;
    const bool negative = (code & sign_bit) != 0;
    float v;
    if (d.nan_code != -1 && (d.nan_signed != 0 ? mag == d.nan_code : code == d.nan_code)) {
      v = NAN;
    } else if (d.inf_code != -1 && mag == d.inf_code) {
      v = INFINITY;
    } else if (mag > d.max_code || (mag == 0 && negative && d.neg_zero == 0)) {
      v = NAN;   // an encoding the format leaves unused
    } else {
      const int e = mag >> (P - 1), frac = mag & ((1 << (P - 1)) - 1);
      v = e == 0 ? ldexpf((float)frac, 2 - P - B) : ldexpf((float)(frac + (1 << (P - 1))), e - B - (P - 1));
    }
    t->v[byte] = negative ? -v : v;
  }
}

// The addend constants of a rounding mode in a code space with `frac` fraction bits.
bool derive_mode8(int variant, int nbits, int max_nbits, fbsr::Mode8* m, uint32_t frac = 24) {
  const bool draws = variant == FBSR_SRFF || variant == FBSR_SRF || variant == FBSR_SRC || variant == FBSR_SRC_TIES_ODD;
  if (variant < FBSR_RNE || variant > FBSR_RNA) return false;
  if (draws && (nbits < 1 || nbits > max_nbits)) return false;
  m->nbits = draws ? (uint32_t)nbits : 0u;
  m->shift = frac - m->nbits;
  m->srf = variant == FBSR_SRF;
  const uint32_t half = m->shift >= 1u ? 1u << (m->shift - 1) : 0u;   // half of the last kept place
  m->tie_xor = (variant == FBSR_SRC_TIES_ODD || variant == FBSR_RNO) ? 1u : 0u;
  m->ties = variant == FBSR_RNE || variant == FBSR_RNO || variant == FBSR_SRC || variant == FBSR_SRC_TIES_ODD;
  m->fixed = m->ties ? (half != 0u ? half - 1u : 0u) : (variant == FBSR_SRF || variant == FBSR_RNA) ? half : 0u;
  return true;
}

struct NamedFormat8 {
  const char* name;
  fbsr_format8 f;
};

// Published formats: OCP 8-bit floating point, OCP microscaling element types.
const NamedFormat8 kNamed[] = {
    {"ocp_e4m3", {8, 4, 7, 0x7E, -1, 0x7F, 1, 1}},
    {"ocp_e5m2", {8, 3, 15, 0x7B, 0x7C, 0x7E, 1, 1}},
    {"ocp_e3m2", {6, 3, 3, 0x1F, -1, -1, 0, 1}},
    {"ocp_e2m3", {6, 4, 1, 0x1F, -1, -1, 0, 1}},
    {"ocp_e2m1", {4, 2, 1, 0x07, -1, -1, 0, 1}},
    {"ieee_binary16", {16, 11, 15, 0x7BFF, 0x7C00, 0x7E00, 1, 1}},
};

}  // namespace

extern "C" {

int fbsr_round(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
               uint64_t offset, void* stream) {
  if (!valid_fmt(fmt)) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset, FBSR_MAX_NBITS_ROUND);
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
  if (!is_8bit_fmt(fmt)) return FBSR_EINVAL;
  if (src_fmt != FBSR_SRC_BF16 && src_fmt != FBSR_SRC_FP16) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset, FBSR_MAX_NBITS_ROUND);
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
  if (!is_8bit_fmt(fmt)) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset, FBSR_MAX_NBITS_ROUND);
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
  if (!is_8bit_fmt(fmt)) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset);
  if (c != FBSR_OK) return c;
  if (p == nullptr) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (w8 == nullptr || g16 == nullptr || m16 == nullptr || v16 == nullptr) return FBSR_EINVAL;
  if (misaligned(g16, 2) || misaligned(m16, 2) || misaligned(v16, 2)) return FBSR_EALIGN;
  fbsr::AdamWScalars sc = {p->lr, p->beta1, p->beta2, p->eps, p->weight_decay, p->bias_corr1, p->bias_corr2, 0.0f, 0.0f, 0};
  fbsr::derive_adamw(&sc);
  const hipError_t e = fbsr::launch_qat_adamw(reinterpret_cast<uint8_t*>(w8), reinterpret_cast<const uint16_t*>(g16),
                                              reinterpret_cast<uint16_t*>(m16), reinterpret_cast<uint16_t*>(v16), n, fmt,
                                              sc, variant, nbits, seed, step, offset,
                                              reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_format8_named(const char* name, fbsr_format8* out) {
  if (name == nullptr || out == nullptr) return FBSR_EINVAL;
  for (const NamedFormat8& k : kNamed) {
    if (strcmp(name, k.name) == 0) {
      *out = k.f;
      return FBSR_OK;
    }
  }
  // IEEE WG P3109 interim report, binary8pP: bias 2^(7-P), NaN 0x80, infinities 0x7F / 0xFF, no -0
  const char* stem = "p3109_binary8p";
  const size_t len = strlen(stem);
  if (strncmp(name, stem, len) == 0 && name[len] >= '1' && name[len] <= '7' && name[len + 1] == '\0') {
    const int P = name[len] - '0';
    *out = fbsr_format8{8, P, 1 << (7 - P), 0x7E, 0x7F, 0x80, 0, 0};
    return FBSR_OK;
  }
  return FBSR_EINVAL;
}

int fbsr_format8_check(const fbsr_format8* fmt) {
  fbsr::Fmt8 f;
  return fmt != nullptr && derive_format8(*fmt, &f) ? FBSR_OK : FBSR_EINVAL;
}

int fbsr_round_format8(const void* x, int src, void* out, uint64_t n, const fbsr_format8* fmt, int variant, int nbits,
                       uint64_t seed, uint64_t offset, void* stream) {
  fbsr::Fmt8 f;
  fbsr::Mode8 m;
  if (fmt == nullptr || !derive_format8(*fmt, &f) || !derive_mode8(variant, nbits, FBSR_MAX_NBITS_ROUND, &m)) return FBSR_EINVAL;
  if (src != FBSR_FROM_BF16 && src != FBSR_FROM_FP16 && src != FBSR_FROM_FP32) return FBSR_EINVAL;
  if (n > fbsr::kMaxElems || offset > UINT64_MAX - n) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (x == nullptr || out == nullptr) return FBSR_EINVAL;
  if (misaligned(x, src == FBSR_FROM_FP32 ? 4 : 2)) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_round_format8(x, src, reinterpret_cast<uint8_t*>(out), n, f, m, seed, offset,
                                                  reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_format16_check(const fbsr_format8* fmt) {
  fbsr::Fmt8 f;
  return fmt != nullptr && derive_format8(*fmt, &f, 16) ? FBSR_OK : FBSR_EINVAL;
}

int fbsr_round_format16(const void* x, int src, void* out, uint64_t n, const fbsr_format8* fmt, int variant, int nbits,
                        uint64_t seed, uint64_t offset, void* stream) {
  fbsr::Fmt8 f;
  fbsr::Mode8 m;
  if (fmt == nullptr || !derive_format8(*fmt, &f, 16)) return FBSR_EINVAL;
  // the last place of n must stay two bits above the end of the code space: one for the half step / the tie position of
  // the inner rounding, one for the sticky bit of a truncated target-subnormal input
  const int max_nbits = (int)f.frac - 2 < FBSR_MAX_NBITS ? (int)f.frac - 2 : FBSR_MAX_NBITS;
  if (!derive_mode8(variant, nbits, max_nbits, &m, f.frac)) return FBSR_EINVAL;
  if (src != FBSR_FROM_BF16 && src != FBSR_FROM_FP16 && src != FBSR_FROM_FP32) return FBSR_EINVAL;
  if (n > fbsr::kMaxElems || offset > UINT64_MAX - n) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (x == nullptr || out == nullptr) return FBSR_EINVAL;
  if (misaligned(x, src == FBSR_FROM_FP32 ? 4 : 2) || misaligned(out, 2)) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_round_format16(x, src, reinterpret_cast<uint16_t*>(out), n, f, m, seed, offset,
                                                   reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_qat_adamw_step_format8(void* w8, const void* g16, void* m16, void* v16, uint64_t n, const fbsr_format8* fmt,
                                const fbsr_adamw* p, int variant, int nbits, uint64_t seed, uint64_t step, uint64_t offset,
                                void* stream) {
  fbsr::Fmt8 f;
  fbsr::Mode8 m;
  if (fmt == nullptr || !derive_format8(*fmt, &f) || !derive_mode8(variant, nbits, FBSR_MAX_NBITS, &m)) return FBSR_EINVAL;
  if (n > fbsr::kMaxElems || offset > UINT64_MAX - n) return FBSR_EINVAL;
  if (p == nullptr) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (w8 == nullptr || g16 == nullptr || m16 == nullptr || v16 == nullptr) return FBSR_EINVAL;
  if (misaligned(g16, 2) || misaligned(m16, 2) || misaligned(v16, 2)) return FBSR_EALIGN;
  fbsr::Table8 t;
  decode_table8(*fmt, &t);
  fbsr::AdamWScalars sc = {p->lr, p->beta1, p->beta2, p->eps, p->weight_decay, p->bias_corr1, p->bias_corr2, 0.0f, 0.0f, 0};
  fbsr::derive_adamw(&sc);
  const hipError_t e = fbsr::launch_qat_adamw_format8(reinterpret_cast<uint8_t*>(w8), reinterpret_cast<const uint16_t*>(g16),
                                                      reinterpret_cast<uint16_t*>(m16), reinterpret_cast<uint16_t*>(v16), n, f,
                                                      m, t, sc, seed, step, offset, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

uint64_t fbsr_bias_stats_workspace_bytes(uint64_t n, uint32_t nbins) {
  (void)nbins;
  return fbsr::stats_workspace_bytes(n);   // two records per chunk of the vector kernel
}

}  // extern "C"

namespace {

// The checks fbsr_bias_stats and fbsr_bias_stats_static share (everything but the workspace).
int check_stats(const float* x, const void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t offset,
                uint64_t group, uint64_t first_bin, uint32_t nbins, const double* stats, bool* nothing_to_do) {
  *nothing_to_do = false;
  if (!valid_fmt(fmt)) return FBSR_EINVAL;
  const int c = check_common(variant, nbits, n, offset, FBSR_MAX_NBITS_ROUND);
  if (c != FBSR_OK) return c;
  if (group == 0 || group > ((uint64_t)1 << 62)) return FBSR_EINVAL;
  if (n == 0) {
    *nothing_to_do = true;
    return FBSR_OK;
  }
  if (x == nullptr || stats == nullptr) return FBSR_EINVAL;
  if (misaligned(x, 4) || misaligned(stats, 8)) return FBSR_EALIGN;
  if (out != nullptr && misaligned(out, code_bytes(fmt))) return FBSR_EALIGN;
  const uint64_t bin_lo = offset / group, bin_hi = (offset + n - 1) / group;
  if (bin_lo < first_bin || bin_hi - first_bin >= nbins) return FBSR_ERANGE;
  return FBSR_OK;
}

}  // namespace

extern "C" {

int fbsr_bias_stats(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
                    uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins, double* stats,
                    void* workspace, uint64_t workspace_bytes, void* stream) {
  bool nothing = false;
  const int c = check_stats(x, out, n, fmt, variant, nbits, offset, group, first_bin, nbins, stats, &nothing);
  if (c != FBSR_OK || nothing) return c;
  if (workspace == nullptr) return FBSR_EINVAL;
  if (misaligned(workspace, 8)) return FBSR_EALIGN;
  if (workspace_bytes < fbsr_bias_stats_workspace_bytes(n, nbins)) return FBSR_ERANGE;
  const hipError_t e =
      fbsr::launch_stats(x, out, n, fmt, variant, nbits, seed, offset, group, first_bin, nbins, stats,
                         reinterpret_cast<double*>(workspace), reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_bias_stats_static(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits, uint64_t seed,
                           uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins, double* stats,
                           void* stream) {
  bool nothing = false;
  const int c = check_stats(x, out, n, fmt, variant, nbits, offset, group, first_bin, nbins, stats, &nothing);
  if (c != FBSR_OK || nothing) return c;
  if (n > fbsr::kStaticMaxElems || fbsr_bias_stats_workspace_bytes(n, nbins) > fbsr::kStaticScratchBytes) return FBSR_ERANGE;
  double* ws = nullptr;
  if (fbsr::static_scratch(&ws) != hipSuccess) return FBSR_EDEVICE;
  // every record finalize reads is written by this call's own tile kernel first: nothing has to start at zero
  const hipError_t e = fbsr::launch_stats(x, out, n, fmt, variant, nbits, seed, offset, group, first_bin, nbins, stats, ws,
                                          reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_bias_stats_format8(const float* x, void* out, uint64_t n, const fbsr_format8* fmt, int variant, int nbits,
                            uint64_t seed, uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins, double* stats,
                            void* workspace, uint64_t workspace_bytes, void* stream) {
  fbsr::Fmt8 f;
  fbsr::Mode8 m;
  if (fmt == nullptr || !derive_format8(*fmt, &f) || !derive_mode8(variant, nbits, FBSR_MAX_NBITS_ROUND, &m)) return FBSR_EINVAL;
  if (n > fbsr::kMaxElems || offset > UINT64_MAX - n) return FBSR_EINVAL;
  if (group == 0 || group > ((uint64_t)1 << 62)) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (x == nullptr || stats == nullptr || workspace == nullptr) return FBSR_EINVAL;
  if (misaligned(x, 4) || misaligned(stats, 8) || misaligned(workspace, 8)) return FBSR_EALIGN;
  const uint64_t bin_lo = offset / group, bin_hi = (offset + n - 1) / group;
  if (bin_lo < first_bin || bin_hi - first_bin >= nbins) return FBSR_ERANGE;
  if (workspace_bytes < fbsr_bias_stats_workspace_bytes(n, nbins)) return FBSR_ERANGE;
  fbsr::Table8 t;
  decode_table8(*fmt, &t);
  const hipError_t e = fbsr::launch_stats_format8(x, reinterpret_cast<uint8_t*>(out), n, f, m, t, fmt->precision, fmt->bias, seed, offset, group,
                                                  first_bin, stats, reinterpret_cast<double*>(workspace),
                                                  reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_probe_stream41(const float* x, void* out, uint64_t n, void* stream) {
  if (n > fbsr::kMaxElems || n % fbsr::kRoundTileElems != 0) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (x == nullptr || out == nullptr) return FBSR_EINVAL;
  if (misaligned(x, 16) || misaligned(out, 4)) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_stream41(x, reinterpret_cast<uint8_t*>(out), n / fbsr::kRoundTileElems,
                                             reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_probe_stream75(void* w8, const void* g16, void* m16, void* v16, uint64_t n, void* stream) {
  if (n > fbsr::kMaxElems || n % fbsr::kTileElems != 0) return FBSR_EINVAL;
  if (n == 0) return FBSR_OK;
  if (w8 == nullptr || g16 == nullptr || m16 == nullptr || v16 == nullptr) return FBSR_EINVAL;
  if (misaligned(w8, 8) || misaligned(g16, 16) || misaligned(m16, 16) || misaligned(v16, 16)) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_stream75(reinterpret_cast<uint8_t*>(w8), reinterpret_cast<const uint16_t*>(g16),
                                             reinterpret_cast<uint16_t*>(m16), reinterpret_cast<uint16_t*>(v16),
                                             n / fbsr::kTileElems, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_check_qat_division(const float* num, const float* den, uint64_t count, uint64_t* counts, void* stream) {
  if (count > fbsr::kMaxElems) return FBSR_EINVAL;
  if (count == 0) return FBSR_OK;
  if (num == nullptr || den == nullptr || counts == nullptr) return FBSR_EINVAL;
  if (misaligned(num, 4) || misaligned(den, 4) || misaligned(counts, 8)) return FBSR_EALIGN;
  const hipError_t e = fbsr::launch_check_division(num, den, count, reinterpret_cast<unsigned long long*>(counts),
                                                   reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

int fbsr_check_qat_root(float bias_corr2, uint64_t* counts, void* stream) {
  if (counts == nullptr || !(bias_corr2 >= 0x1p-20f && bias_corr2 <= 1.0f)) return FBSR_EINVAL;
  if (misaligned(counts, 8)) return FBSR_EALIGN;
  fbsr::AdamWScalars sc = {};
  sc.bias_corr1 = 1.0f;
  sc.bias_corr2 = bias_corr2;
  sc.eps = 1e-8f;
  fbsr::derive_adamw(&sc);
  const hipError_t e = fbsr::launch_check_corrected_root(sc, reinterpret_cast<unsigned long long*>(counts),
                                                         reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? FBSR_OK : FBSR_EDEVICE;
}

const char* fbsr_strerror(int status) {
  switch (status) {
    case FBSR_OK: return "ok";
    case FBSR_EINVAL: return "invalid argument";
    case FBSR_EALIGN: return "pointer not aligned to its element type";
    case FBSR_ERANGE: return "element outside the bins, workspace too small, or call too large for the built-in workspace";
    case FBSR_EDEVICE: return "HIP runtime error at launch";
  }
  return "unknown status";
}

int fbsr_version(void) { return 101; }

}  // extern "C"
