/* CPU check of the short division used by the fused QAT kernel for x / c with a bf16-valued x and a divisor c
 * that is uniform over the launch:
 *     r = RN(1 / c);  q = RN(x r);  t = fma(q, c, -x);  result = fma(-t, r, q)
 * Claim: the result is the correctly rounded quotient RN(x / c), signed zeros included, for every c in [2^-20, 1]
 * and every x that is zero or has |x| >= 2^-103; an overflowing quotient or a non-finite x gives the same infinity
 * or a NaN (which the kernel treats as "recompute exactly").  IEEE binary32 arithmetic is the same on the host, so
 * the claim is checked here with fmaf: every bf16 significand against every `stride`-th divisor significand, at
 * the exponents given.  Prints the number of counterexamples. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float from_bits(uint32_t u) { float v; memcpy(&v, &u, 4); return v; }
static uint32_t to_bits(float v) { uint32_t u; memcpy(&u, &v, 4); return u; }

static int same(volatile float x, volatile float c) {
  const float r = 1.0f / c;
  const float q = x * r;
  const float t = fmaf(q, c, -x);
  const float got = fmaf(-t, r, q);
  const float want = x / c;
  return to_bits(got) == to_bits(want) || isnan(got);
}

int main(int argc, char** argv) {
  const uint32_t stride = argc > 1 ? (uint32_t)atoi(argv[1]) : 64;
  const int a_list[] = {-103, -64, 0, 100, 127};
  const int b_list[] = {-20, -1};
  unsigned long long bad = 0, cases = 0;
  for (unsigned ai = 0; ai < sizeof(a_list) / sizeof(int); ++ai)
    for (unsigned bi = 0; bi < sizeof(b_list) / sizeof(int); ++bi)
      for (uint32_t cm = 0; cm < (1u << 23); cm += stride) {
        const float c = from_bits(((uint32_t)(b_list[bi] + 127) << 23) | cm);
        for (uint32_t xm = 0; xm < 128; ++xm)
          for (uint32_t s = 0; s < 2; ++s) {
            bad += !same(from_bits((s << 31) | ((uint32_t)(a_list[ai] + 127) << 23) | (xm << 16)), c);
            ++cases;
          }
      }
  /* c = 1 exactly, zeros of both signs, infinities */
  const float cs[] = {1.0f, 0.1f, 0.001f, 0x1p-20f};
  const uint32_t xs[] = {0x00000000u, 0x80000000u, 0x7F800000u, 0xFF800000u, 0x7F7F0000u, 0xFF7F0000u};
  for (unsigned i = 0; i < 4; ++i)
    for (unsigned j = 0; j < 6; ++j) { bad += !same(from_bits(xs[j]), cs[i]); ++cases; }
  printf("%llu %llu\n", bad, cases);
  return bad != 0;
}
