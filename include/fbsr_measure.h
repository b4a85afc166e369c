/* fbsr_measure.h -- measurement aids of libfbsr.so.  Nothing here belongs to the method of the paper or to the
 * library's product interface (include/fbsr.h): these entry points exist so that a benchmark can time the launch
 * shapes of the kernels with the arithmetic taken out, and so that a test can check on the device the arithmetic
 * identities one kernel relies on. */
#ifndef FBSR_MEASURE_H
#define FBSR_MEASURE_H

#include <stdint.h>

#include "fbsr.h" /* the status codes */

#ifdef __cplusplus
extern "C" {
#endif

/* Streams n floats through the rounding kernels' launch shape with no
 * arithmetic (out[j] = the top byte of x[j]'s pattern): every input byte read once, one byte written per element.
 * Its throughput is the practical ceiling for fbsr_round's 4 : 1 read : write traffic on the part at hand.
 * n must be a multiple of 4096, x 16-byte and out 4-byte aligned (else FBSR_EINVAL / FBSR_EALIGN). */
int fbsr_probe_stream41(const float* x, void* out, uint64_t n, void* stream);

/* Streams n elements through the fused training step's launch shape with no arithmetic: per element one weight byte
 * and three 16-bit words (gradient, both moments) read, the weight byte and both moments written back in place
 * (each combined with the gradient's bits by an exclusive or, so calling it twice restores the buffers).  Its
 * throughput is the practical ceiling for fbsr_qat_adamw_step's 7 : 5 read : write traffic on the part at hand.
 * All four are device pointers; n must be a multiple of 2048, w8 8-byte and the others 16-byte aligned
 * (else FBSR_EINVAL / FBSR_EALIGN). */
int fbsr_probe_stream75(void* w8, const void* g16, void* m16, void* v16, uint64_t n, void* stream);

/* Device self-checks of two arithmetic identities inside fbsr_qat_adamw_step's tile kernel, run with the kernel's own
 * device functions on the part at hand (Alg. 1's AdamW update is evaluated as single correctly rounded fp32
 * operations; the kernel shortens two of them and these calls show that the bits do not change).
 * fbsr_check_qat_division: counts[0] += the number of pairs k < count for which the kernel's division of num[k] by
 *   den[k] without operand scaling differs from the correctly rounded quotient (its NaN counts as agreement: the kernel
 *   then recomputes with the full division).  Meant for den in [2^-28, 2^65) and |num| zero or at least 2^-40.
 * fbsr_check_qat_root: counts[1] += the number of bf16 second-moment codes (all 65536) for which the root read from the
 *   kernel's two tables differs from sqrt(v / bias_corr2) (a NaN from the tables counts as agreement; for codes below
 *   2^-125 the tables read zero and the root must be below 2^-52).  bias_corr2 in [2^-20, 1] (else FBSR_EINVAL).
 * num, den: device, 4-byte aligned.  counts: two 64-bit counters on the device, 8-byte aligned, accumulated into. */
int fbsr_check_qat_division(const float* num, const float* den, uint64_t count, uint64_t* counts, void* stream);
int fbsr_check_qat_root(float bias_corr2, uint64_t* counts, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FBSR_MEASURE_H */
