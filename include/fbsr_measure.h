/* fbsr_measure.h -- measurement aids of libfbsr.so.  Nothing here belongs to the method of the paper or to the
 * library's product interface (include/fbsr.h): these entry points exist so that a benchmark can time the launch
 * shapes of the kernels with the arithmetic taken out. */
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
 * n must be a multiple of 2048, x 16-byte and out 4-byte aligned (else FBSR_EINVAL / FBSR_EALIGN). */
int fbsr_probe_stream41(const float* x, void* out, uint64_t n, void* stream);

/* Streams n elements through the fused training step's launch shape with no arithmetic: per element one weight byte
 * and three 16-bit words (gradient, both moments) read, the weight byte and both moments written back in place
 * (each combined with the gradient's bits by an exclusive or, so calling it twice restores the buffers).  Its
 * throughput is the practical ceiling for fbsr_qat_adamw_step's 7 : 5 read : write traffic on the part at hand.
 * All four are device pointers; n must be a multiple of 2048, w8 8-byte and the others 16-byte aligned
 * (else FBSR_EINVAL / FBSR_EALIGN). */
int fbsr_probe_stream75(void* w8, const void* g16, void* m16, void* v16, uint64_t n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FBSR_MEASURE_H */
