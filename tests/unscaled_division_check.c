/* CPU check of the division the fused QAT kernel uses for m / (sqrt(v) + eps):
 *     r0 ~ 1 / d (any value within one ulp);  e = fma(-d, r0, 1);  r = fma(e, r0, r0);
 *     q = RN(n r);  q = fma(fma(-d, q, n), r, q), twice
 * i.e. the operations of the usual correctly rounded division sequence without its scaling of extreme operands.
 * Claim: for d in [2^-28, 2^65) and |n| in [2^-40, 2^101) with a finite quotient the result is RN(n / d) from EVERY
 * start r0 within one ulp of 1 / d -- with one exception that no such sequence can avoid: a divisor whose significand
 * is all ones together with the start just BELOW the correctly rounded reciprocal (the Newton step then ties back to
 * the start).  The device's reciprocal instruction is on the right side there, or its ordinary division would be
 * wrong too; a test on the device checks exactly those operands.  IEEE binary32 arithmetic is the same on the host,
 * so the claim is checked here with fmaf on operand pairs drawn to favour all-ones and all-zeros significands.
 * Prints: counterexamples outside the exception, cases inside it, cases tried. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float from_bits(uint32_t u) { float v; memcpy(&v, &u, 4); return v; }
static uint32_t to_bits(float v) { uint32_t u; memcpy(&u, &v, 4); return u; }

static float short_division(float n, float d, float r0) {
  const float e = fmaf(-d, r0, 1.0f);
  const float r = fmaf(e, r0, r0);
  float q = n * r;
  q = fmaf(fmaf(-d, q, n), r, q);
  q = fmaf(fmaf(-d, q, n), r, q);
  return q;
}

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t next(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return state; }

int main(int argc, char** argv) {
  const uint64_t draws = argc > 1 ? strtoull(argv[1], 0, 10) : 20000000ull;
  uint64_t bad = 0, corner = 0, cases = 0;
  for (uint64_t i = 0; i < draws; ++i) {
    const uint64_t a = next(), b = next();
    uint32_t md = (uint32_t)a & 0x7FFFFFu, mn = (uint32_t)(a >> 32) & 0x7FFFFFu;
    switch ((b >> 60) & 7) {
      case 0: md = 0x7FFFFFu - (uint32_t)((b >> 40) & 3); break;
      case 1: md = (uint32_t)((b >> 40) & 3); break;
      case 2: mn &= 0x7F0000u; break;
      case 3: mn = 0; md = 0x7FFFFFu - (uint32_t)((b >> 40) & 7); break;
      default: break;
    }
    const int ed = -28 + (int)((b & 0xFFFF) % 93);            /* d in [2^-28, 2^65) */
    const int en = -40 + (int)(((b >> 16) & 0xFFFF) % 141);   /* |n| in [2^-40, 2^101) */
    if (en - ed > 126) continue;                              /* the quotient overflows */
    const float d = from_bits(((uint32_t)(ed + 127) << 23) | md);
    float n = from_bits(((uint32_t)(en + 127) << 23) | mn);
    if ((b >> 59) & 1) n = -n;
    const float want = n / d, rc = 1.0f / d;
    for (int k = -1; k <= 1; ++k) {
      const float r0 = from_bits(to_bits(rc) + (uint32_t)k);
      const double ulp = (double)from_bits(to_bits(rc) & 0x7F800000u) * 1.1920928955078125e-7;
      if (fabs((double)r0 - 1.0 / (double)d) > ulp) continue;   /* not within one ulp of the true reciprocal */
      ++cases;
      if (to_bits(short_division(n, d, r0)) != to_bits(want)) {
        if (md == 0x7FFFFFu && k == -1) ++corner;
        else ++bad;
      }
    }
  }
  printf("%llu %llu %llu\n", (unsigned long long)bad, (unsigned long long)corner, (unsigned long long)cases);
  return bad != 0;
}
