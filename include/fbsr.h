/* fbsr.h -- few-bit stochastic rounding (FBSR) on AMD MI355X (gfx950), C ABI.
 *
 * Implements the elementwise hot path of "On Stochastic Rounding with Few Random Bits"
 * (arXiv 2504.20634): fp32 values are rounded to a narrower binary format using only
 * N random bits per element.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library allocates and
 *     frees nothing, enqueues its kernels on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and returns without synchronising.
 *   - The return value is an fbsr_status; nothing throws or aborts.  Argument errors are
 *     detected on the host before anything is launched (so they can be tested without a GPU).
 *   - n == 0 is FBSR_OK and launches nothing.  n may be at most 2^38 elements and offset + n must
 *     not overflow 64 bits (else FBSR_EINVAL); large calls are cut into several launches.
 *   - Results are a pure function of the arguments: the random bits of an element depend only
 *     on (seed, step, global element index), so repeating a call, or cutting it into chunks
 *     whose `offset` continues the index, gives identical bytes.
 *   - Random bits (the paper leaves the source open, Sec. II-B): Philox4x32-10 with
 *     key = (seed lo, seed hi) and counter = (block lo, block hi, step lo, step hi).  With
 *     W = the smallest power of two >= nbits, a 128-bit block (word 0 = bits 0..31) is cut
 *     into 128/W slots; element i uses the low nbits bits of slot i mod (128/W) of block
 *     floor(i / (128/W)).  So one block serves 128/W elements.
 *   - Formats follow the (K, P, B; M) model of Sec. II, Eq. (1); codes are the packed
 *     sign | exponent | trailing-significand bits.
 *   - Alignment: x / g need 4-byte, bf16 codes 2-byte alignment (else FBSR_EALIGN).  The
 *     vectorised kernels are used when x is 16-byte aligned at the first element whose
 *     global index is a multiple of 128/W and the output is aligned accordingly; otherwise,
 *     and for ragged heads and tails, a slower per-element kernel gives the same bytes.
 */
#ifndef FBSR_H
#define FBSR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Target formats (Sec. II).  Codes are uint16 for BF16, uint8 for the 8-bit formats. */
typedef enum {
  FBSR_FMT_BF16 = 0,     /* K=16 P=8 B=127, M=(2-2^-7)*2^127, has infinities               */
  FBSR_FMT_E4M3 = 1,     /* OCP E4M3: K=8 P=4 B=7, M=448, no infinities, S.1111.111 is NaN  */
  FBSR_FMT_E5M2 = 2,     /* OCP E5M2: K=8 P=3 B=15, M=57344, has infinities                 */
  FBSR_FMT_BINARY8P4 = 3 /* IEEE WG P3109 (interim report) binary8p4, the format Sec. IV trains in: K=8 P=4 B=8,
                            M=224, infinities 0x7F / 0xFF, 0x80 the only NaN, no negative zero.  Rounded by the
                            rules of fbsr_round_format8 under the descriptor "p3109_binary8p4": above M nearest
                            even (the tie 232 stays at M, anything above goes to infinity), NaN -> 0x80 whatever
                            its sign, a negative input that rounds to zero -> 0x00                             */
} fbsr_fmt;

/* Rounding predicates (delta = fractional part of the scaled significand, Sec. II-A Eq. (5);
 * n = the element's nbits-bit random integer; N = nbits).                                    */
typedef enum {
  FBSR_RNE = 0,  /* round to nearest, ties to even (Sec. II-A); nbits ignored, no random bits */
  FBSR_SRFF = 1, /* delta + n 2^-N >= 1             (Sec. II-B; biased by -2^-(N+1) ulp)      */
  FBSR_SRF = 2,  /* delta + (n + 1/2) 2^-N >= 1     (Sec. II-B)                               */
  FBSR_SRC = 3   /* SRFF on Round(delta 2^N) 2^-N, Round = nearest, ties to even (Eq. (7))    */
} fbsr_variant;

typedef enum {
  FBSR_OK = 0,
  FBSR_EINVAL = 1,  /* bad enum, nbits outside [1, the entry point's maximum], null pointer, group == 0, ... */
  FBSR_EALIGN = 2,  /* a pointer is not aligned to its element type                              */
  FBSR_ERANGE = 3,  /* an element would fall outside the caller's bins / workspace too small / call too
                       large for fbsr_bias_stats_static                                          */
  FBSR_EDEVICE = 4  /* the HIP runtime reported an error at launch                               */
} fbsr_status;

/* Largest nbits.  Every entry point but the fused updates and the 16-bit-code one (fbsr_round, fbsr_round_from16,
 * fbsr_round_format8, fbsr_round_block_scaled, fbsr_bias_stats, fbsr_bias_stats_format8) takes up to
 * FBSR_MAX_NBITS_ROUND, which covers every
 * bit an fp32 source can drop towards an 8-bit target (D = 20 for E4M3 and binary8p4, 21 for E5M2), so that nbits >= D
 * gives classical SR; calls with more than FBSR_MAX_NBITS bits use 32-bit slots (4 elements per Philox block), where
 * the generator's cost per element is four times that of 8-bit slots.  The fused updates take up to FBSR_MAX_NBITS: their rounding drops at
 * most 16 bits of a normal result (fp32 -> bf16 in fbsr_sgd_update, a bf16 sum -> 8 bits in the QAT steps), so 16
 * bits already are classical SR there. */
#define FBSR_MAX_NBITS 16
#define FBSR_MAX_NBITS_ROUND 24

/* 16-bit source formats of fbsr_round_from16. */
typedef enum {
  FBSR_SRC_BF16 = 0, /* K=16 P=8  B=127 */
  FBSR_SRC_FP16 = 1  /* IEEE binary16: K=16 P=11 B=15 */
} fbsr_src16;

/* Rounds n fp32 values to `fmt`:  out[j] = FBSR(x[j]; bits of global element offset + j,
 * stream (seed, step = 0)).
 *   Sign-magnitude: |x| is rounded and the sign re-applied (the paper rounds positive values),
 *   so "up" is away from zero.  +-0 -> +-0.  NaN -> canonical quiet NaN with x's sign
 *   (bf16 0x7FC0, E5M2 0x7E, E4M3 0x7F).  |x| > M is rounded deterministically (Sec. II):
 *   bf16 / E5M2 to M below M + ulp(M)/2 and to infinity from there on, E4M3 saturates to +-M.
 *   Target subnormals are rounded on the subnormal grid (Eq. (2): the exponent is clamped at
 *   1 - B); fp32 subnormal inputs are ordinary values.
 * x: n floats (device, read).  out: n codes (device, written; must not overlap x).
 * Errors: FBSR_EINVAL (bad fmt / variant / nbits, null pointer with n > 0), FBSR_EALIGN,
 * FBSR_EDEVICE. */
int fbsr_round(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits,
               uint64_t seed, uint64_t offset, void* stream);

/* Narrow-source rounding, the paper's own setting (Sec. III-E: inputs of precision Q = P + D with
 * few excess bits D; Fig. 2: bf16 -> a precision-3 target, D = 5; Sec. IV: bf16 updates -> an 8-bit
 * format): out[j] = FBSR(value of x[j]) exactly as fbsr_round, with the 16-bit source value taken
 * exactly (bf16 -> E4M3 has D = 4, bf16 -> E5M2 D = 5, binary16 -> E4M3 D = 7, binary16 -> E5M2
 * D = 8).  nbits may exceed D; all variants then coincide with exact SR (App. A-C).
 * x: n 16-bit codes of src_fmt (device, read, 2-byte aligned).  out: n fp8 codes (device, written).
 * fmt must be one of the 8-bit formats (else FBSR_EINVAL).  Other errors as fbsr_round. */
int fbsr_round_from16(const void* x, void* out, uint64_t n, int src_fmt, int fmt, int variant, int nbits,
                      uint64_t seed, uint64_t offset, void* stream);

/* The weight update of Alg. 1 ("w <- RoundTo(w + u), SR applied here") fused into one pass,
 * in SGD form:  w[j] <- FBSR_bf16( fma(-lr, g[j], float(w[j])) )  with the bits of
 * (seed, step, offset + j).  The fma is a single-rounding fp32 fused multiply-add with IEEE
 * subnormals.
 * w: n bf16 codes (device, updated in place).  g: n floats (device, read).
 * Errors as fbsr_round. */
int fbsr_sgd_update(void* w, const float* g, uint64_t n, float lr, int variant, int nbits,
                    uint64_t seed, uint64_t step, uint64_t offset, void* stream);

/* Elements per shared scale in fbsr_round_block_scaled. */
#define FBSR_SCALE_BLOCK 32

/* Block-scaled fp8 target (Sec. I-A: "blocks of low-precision values are accompanied by a scale factor,
 * which may be a power of two"; the paper fixes no rule for it).  Blocks of FBSR_SCALE_BLOCK consecutive
 * elements of the call (element j belongs to block j / 32; the last block may be short) share the scale
 * 2^s,  s = clamp(floor(log2 amax) - emax, -127, 127),  amax = max |x| over the block,
 * emax = floor(log2 M) of the element format (8 for E4M3, 15 for E5M2);  scales[b] = s + 127.
 * Every element is out[j] = FBSR_fmt(x[j] * 2^-s) (an exact scaling) with the random bits of global index
 * offset + j, as in fbsr_round; the block's largest element lands in [2^emax, 2^(emax+1)) and whatever
 * exceeds M there follows fbsr_round's out-of-range rule.  A block of zeros has s = -127.  A block that
 * holds a NaN or an infinity gets scales[b] = 0xFF and all its elements the positive canonical NaN.
 * x: n floats (device, read).  out: n fp8 codes (device, written).  scales: ceil(n / 32) bytes (device,
 * written).  fmt must be one of the 8-bit formats (emax = 7 for binary8p4, whose elements above M follow its own
 * out-of-range rule).  Errors as fbsr_round. */
int fbsr_round_block_scaled(const float* x, void* out, void* scales, uint64_t n, int fmt, int variant,
                            int nbits, uint64_t seed, uint64_t offset, void* stream);

/* Scalars of one AdamW step (decoupled weight decay).  bias_corr1 = 1 - beta1^t and
 * bias_corr2 = 1 - beta2^t for the step count t >= 1 are supplied by the caller. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay, bias_corr1, bias_corr2;
} fbsr_adamw;

/* One fused step of Alg. 1 (quantization-aware training of an 8-bit model with 16-bit updates):
 *   w16 <- w8;  u16 <- AdamW update in 16-bit;  w8 <- RoundTo8(w16 + u16), SR applied to that rounding.
 * The 16-bit format is bf16 (Sec. IV computes the updates in BFloat16).  Per element, every step is one
 * IEEE fp32 operation (round to nearest even, subnormals kept) in this order, and every quantity the
 * listing types as F16 is rounded to bf16 with ties to even:
 *   m  <- bf16( fma(beta1, m, (1 - beta1) * g) )          v <- bf16( fma(beta2, v, (1 - beta2) * (g * g)) )
 *   r  =  (m / bias_corr1) / (sqrt(v / bias_corr2) + eps)     (with the new bf16 m and v)
 *   u  <- bf16( -lr * fma(weight_decay, w, r) )            s <- bf16( w + u )
 *   w8 <- FBSR_fmt(s)  with the random bits of (seed, step, offset + j), as in fbsr_round_from16.
 * So the value handed to the 8-bit rounding has bf16 precision: D = 4 excess bits for E4M3 (the count
 * Sec. IV reasons with), 5 for E5M2.  A NaN produced anywhere is stored as the positive canonical NaN.
 * w8: n codes of fmt (an 8-bit format; device, updated in place).  g16: n bf16 gradients (device, read).
 * m16, v16: n bf16 moments (device, updated in place).  p: HOST pointer, read during the call.
 * Errors: FBSR_EINVAL (fmt not fp8, bad variant / nbits, null pointer), FBSR_EALIGN (16-bit arrays need
 * 2-byte alignment), FBSR_EDEVICE. */
int fbsr_qat_adamw_step(void* w8, const void* g16, void* m16, void* v16, uint64_t n, int fmt,
                        const fbsr_adamw* p, int variant, int nbits, uint64_t seed, uint64_t step,
                        uint64_t offset, void* stream);

/* Rounds as fbsr_round and reduces the rounding error per bin -- the measurement behind
 * Figs. 1 and 2 (mean of the rounded samples per input value; bias = mean of rounded minus
 * input, Sec. III).  Element j has global index i = offset + j and bin
 * floor(i / group) - first_bin, which must lie in [0, nbins) for every element
 * (else FBSR_ERANGE).
 * stats: nbins x 4 doubles {count, sum y, sum e, sum e^2} (device), ACCUMULATED into (the
 *   caller zeroes them), where y is the decoded rounded value and e = (y - x) / ulp_t(x) with
 *   ulp_t(x) = 2^(e~ - P + 1), e~ = max(floor(log2 |x|), 1 - B) (Eq. (2)), all in fp64.
 *   Non-finite x or y propagate through the sums by IEEE rules.  The summation order is fixed,
 *   so repeated calls give identical bits.
 * out: n codes as in fbsr_round, or NULL to skip writing them.
 * workspace: device scratch of at least fbsr_bias_stats_workspace_bytes(n, nbins) bytes,
 *   8-byte aligned, contents irrelevant before and after (else FBSR_ERANGE / FBSR_EALIGN).
 * Two calls that accumulate into the same stats must be ordered on the stream. */
int fbsr_bias_stats(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits,
                    uint64_t seed, uint64_t offset, uint64_t group, uint64_t first_bin,
                    uint32_t nbins, double* stats, void* workspace, uint64_t workspace_bytes,
                    void* stream);

/* fbsr_bias_stats for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc) and so have no workspace to pass: the same kernels, with the workspace
 * in a fixed 1 MiB array inside the library's device image (each GPU the library runs on holds it until the
 * process ends).  The call allocates and frees nothing.  n may be at most FBSR_BIAS_STATS_STATIC_MAX_ELEMS
 * (else FBSR_ERANGE); everything else -- arguments, results bit for bit, errors -- as fbsr_bias_stats.
 * All calls on one GPU share that array: two of them must not overlap in time (order them on one stream, or
 * synchronise between them), or they race.  Nothing in it has to be cleared between calls. */
#define FBSR_BIAS_STATS_STATIC_MAX_ELEMS ((uint64_t)1 << 28)
int fbsr_bias_stats_static(const float* x, void* out, uint64_t n, int fmt, int variant, int nbits,
                           uint64_t seed, uint64_t offset, uint64_t group, uint64_t first_bin,
                           uint32_t nbins, double* stats, void* stream);

/* Bytes of workspace fbsr_bias_stats needs for n elements (never 0; independent of nbins
 * today, kept in the signature for layouts that are not). */
uint64_t fbsr_bias_stats_workspace_bytes(uint64_t n, uint32_t nbins);

/* ---------------------------------------------------------------- generic 8-bit-or-narrower targets */

/* Any format (K, P, B; M) of Sec. II, Eq. (1) whose codes fit a byte.  The paper's format model leaves
 * special encodings open, so they are part of the descriptor.
 *   width       K, 2..8: code = sign | exponent (K - P bits) | trailing significand (P - 1 bits)
 *   precision   P, 1..K-1
 *   bias        B, 0..96
 *   max_code    magnitude code (exponent << (P-1) | trailing bits) of M, the largest finite value; M must
 *               be a normal value and M + ulp(M) a finite fp32 value.  Magnitude codes above max_code
 *               are never produced, except inf_code
 *   inf_code    magnitude code of infinity (above max_code), or -1: the format has none and SATURATES,
 *               every |x| > M (infinities included) becomes +-M
 *   nan_code    full code of the canonical NaN, or -1: the format has none and a NaN input becomes +-M.
 *               Its magnitude part must be an unused one (above max_code, not inf_code), or it is the
 *               sign bit alone in a format without negative zero
 *   nan_signed  nonzero: the sign of a NaN input is OR-ed into nan_code (whose own sign bit must be 0)
 *   neg_zero    nonzero: the format has -0.  Otherwise a negative input that rounds to zero gives code 0
 * With an infinity, |x| > M is rounded to nearest on the unbounded-exponent grid, ties to even, whatever
 * the variant (Sec. II: out-of-range values are "rounded deterministically as in IEEE-754 round to
 * nearest"): below M + ulp(M)/2 to M, above it to infinity, the tie to whichever of the two has the even
 * significand. */
typedef struct {
  int32_t width, precision, bias, max_code, inf_code, nan_code, nan_signed, neg_zero;
} fbsr_format8;

/* Source types of fbsr_round_format8 (the first two as in fbsr_src16). */
#define FBSR_FROM_BF16 0
#define FBSR_FROM_FP16 1
#define FBSR_FROM_FP32 2

/* Further rounding predicates, accepted by fbsr_round_format8 only. */
#define FBSR_SRC_TIES_ODD 4 /* Eq. (7) with Round = nearest, ties to odd (Sec. III-F allows either)      */
#define FBSR_RNO 5          /* round to nearest, ties to odd (Sec. II-A, R_TNO); nbits ignored            */
#define FBSR_RNA 6          /* round to nearest, ties away from zero (Eq. (4), R_TA); nbits ignored       */

/* Fills *out with a published format.  Names: "ocp_e4m3", "ocp_e5m2" (OCP 8-bit floating point; the same
 * formats as FBSR_FMT_E4M3 / FBSR_FMT_E5M2), "ocp_e3m2", "ocp_e2m3", "ocp_e2m1" (OCP microscaling element
 * types: no NaN, no infinity), "ieee_binary16" (IEEE 754 binary16, for fbsr_round_format16 only),
 * "p3109_binary8p1" .. "p3109_binary8p7" (IEEE WG P3109 interim report:
 * bias 2^(7-P), 0x80 the only NaN, 0x7F / 0xFF the infinities, no negative zero; binary8p4 is the format
 * Sec. IV trains in).  Host-only.  Returns FBSR_OK, or FBSR_EINVAL for an unknown name or a null pointer. */
int fbsr_format8_named(const char* name, fbsr_format8* out);

/* FBSR_OK when the descriptor satisfies the constraints above, else FBSR_EINVAL.  Host-only. */
int fbsr_format8_check(const fbsr_format8* fmt);

/* Rounds n values of source type src to the format *fmt, one code per output byte (bits above K zero):
 * out[j] = FBSR(value of x[j]; bits of global element offset + j, stream (seed, step = 0)), with the
 * conventions of fbsr_round (sign-magnitude, target subnormals on the clamped-exponent grid of Eq. (2))
 * and the descriptor's treatment of specials.  For the two OCP fp8 descriptors the result equals
 * fbsr_round / fbsr_round_from16 byte for byte.
 * x: n floats (FBSR_FROM_FP32) or n 16-bit codes (device, read).  out: n bytes (device, written).
 * fmt: HOST pointer, read during the call.  variant: FBSR_RNE .. FBSR_RNA.
 * Errors: FBSR_EINVAL (bad descriptor / src / variant / nbits, null pointer), FBSR_EALIGN, FBSR_EDEVICE. */
int fbsr_round_format8(const void* x, int src, void* out, uint64_t n, const fbsr_format8* fmt, int variant,
                       int nbits, uint64_t seed, uint64_t offset, void* stream);

/* fbsr_bias_stats (the measurement behind Figs. 1 and 2, Sec. III) for a target format given by its descriptor and
 * any rounding mode of fbsr_round_format8: per bin {count, sum y, sum e, sum e^2} with y the Eq. (1) value of the
 * rounded code under the descriptor (infinity for the infinity code, NaN for a NaN code) and e = (y - x) / ulp_t(x),
 * ulp_t(x) = 2^(e~ - P + 1), e~ = max(floor(log2 |x|), 1 - B) (Eq. (2)) with the descriptor's P and B.
 * x: n fp32 values (device).  out: n codes, one per byte (device), or NULL.  fmt: HOST pointer, read during the call.
 * nbits up to FBSR_MAX_NBITS_ROUND.  Bins, stats, workspace (fbsr_bias_stats_workspace_bytes), accumulation, the
 * fixed summation order and the errors are those of fbsr_bias_stats; a bad descriptor or mode gives FBSR_EINVAL. */
int fbsr_bias_stats_format8(const float* x, void* out, uint64_t n, const fbsr_format8* fmt, int variant, int nbits,
                            uint64_t seed, uint64_t offset, uint64_t group, uint64_t first_bin, uint32_t nbins,
                            double* stats, void* workspace, uint64_t workspace_bytes, void* stream);

/* The same for formats of up to 16 bits (IEEE binary16 and any other (K, P, B; M) with K <= 16): one code per
 * 16-bit word of out (bits above K zero).  The descriptor is the struct above with width 2..16 and bias 0..127;
 * because an fp32 source drops 24 - P bits and the kernels keep 32 - K fraction bits beside a code, the precision must be
 * at least K - 8 (binary16: P = 11 >= 8).  bf16 itself (whose M + ulp(M) is not a finite fp32 value) is served by
 * fbsr_round, not by a descriptor.  nbits at most min(FBSR_MAX_NBITS, 30 - K) (14 for a 16-bit format): with
 * P >= K - 8 a target-normal fp32 input drops at most 32 - K bits, so every nbits from 24 - P on (13 for binary16)
 * already is classical SR.  "ieee_binary16" is a name fbsr_format8_named knows.
 * out: n 16-bit codes (device, written, 2-byte aligned).  Everything else as fbsr_round_format8. */
int fbsr_format16_check(const fbsr_format8* fmt);
int fbsr_round_format16(const void* x, int src, void* out, uint64_t n, const fbsr_format8* fmt, int variant,
                        int nbits, uint64_t seed, uint64_t offset, void* stream);

/* fbsr_qat_adamw_step with the 8-bit weights in a generic format (Sec. IV trains in P3109 binary8p4 with bf16
 * updates and 3 random bits) and any variant FBSR_RNE .. FBSR_RNA.  The arithmetic is that of
 * fbsr_qat_adamw_step; a weight byte is decoded by Eq. (1) under the descriptor (bits above K ignored; the NaN
 * code and encodings the format leaves unused enter as NaN, the infinity codes as infinities), and
 * w8 <- FBSR_fmt(s) as in fbsr_round_format8.  A NaN sum is stored as the descriptor's NaN code without a
 * sign, or as +M in a format without NaN.  With an OCP fp8 descriptor the results equal fbsr_qat_adamw_step's.
 * fmt and p are HOST pointers, read during the call.  Errors as fbsr_qat_adamw_step / fbsr_round_format8. */
int fbsr_qat_adamw_step_format8(void* w8, const void* g16, void* m16, void* v16, uint64_t n, const fbsr_format8* fmt,
                                const fbsr_adamw* p, int variant, int nbits, uint64_t seed, uint64_t step,
                                uint64_t offset, void* stream);

/* Static description of a status code. */
const char* fbsr_strerror(int status);

/* Library version, major * 100 + minor. */
int fbsr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FBSR_H */
