/* CPU check of the square root used on the fused QAT kernel's main path:
 *     s = an approximation of sqrt(x) within one unit in the last place (the hardware instruction's guarantee);
 *     lo = the binary32 number just below s, hi = the one just above;
 *     s <- lo if fma(-lo, s, x) <= 0;   s <- hi if fma(-hi, s, x) > 0
 * Claim: for every finite x >= 2^-96 the result is the correctly rounded square root whichever approximation
 * within one ulp the first step delivered, and x = +0, -0 and +infinity come back unchanged.  The two residuals
 * are x - lo s and x - hi s rounded once, so their signs say on which side of x the products lie -- provided they
 * do not underflow, which is what the lower limit on x is for.  IEEE binary32 arithmetic is the same on the host,
 * so the claim is checked here with fmaf: every `stride`-th significand at the exponents listed (both parities),
 * each from every starting point within one ulp of the root.  Prints counterexamples and cases. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float from_bits(uint32_t u) { float v; memcpy(&v, &u, 4); return v; }
static uint32_t to_bits(float v) { uint32_t u; memcpy(&u, &v, 4); return u; }

static float corrected(volatile float s, volatile float x) {
  const float lo = from_bits(to_bits(s) - 1u), hi = from_bits(to_bits(s) + 1u);
  const float r_lo = fmaf(-lo, s, x), r_hi = fmaf(-hi, s, x);
  float out = s;
  if (r_lo <= 0.0f) out = lo;
  if (r_hi > 0.0f) out = hi;
  return out;
}

int main(int argc, char** argv) {
  const uint32_t stride = argc > 1 ? (uint32_t)atoi(argv[1]) : 64;
  const int e_list[] = {-96, -95, -60, -1, 0, 1, 2, 63, 126, 127};
  unsigned long long bad = 0, cases = 0;
  for (unsigned ei = 0; ei < sizeof(e_list) / sizeof(int); ++ei)
    for (uint32_t m = 0; m < (1u << 23); m += stride) {
      const float x = from_bits(((uint32_t)(e_list[ei] + 127) << 23) | m);
      const double root = sqrt((double)x);      /* correctly rounded in binary64 */
      const float want = (float)root;            /* and, for a square root of a binary32 number, in binary32 */
      const double ulp = (double)from_bits(to_bits(want) + 1u) - (double)want;
      for (int d = -1; d <= 1; ++d) {
        const float s = from_bits(to_bits(want) + (uint32_t)d);
        if (fabs((double)s - root) >= ulp) continue;   /* not a value the first step may deliver */
        bad += to_bits(corrected(s, x)) != to_bits(want);
        ++cases;
      }
    }
  /* zeros and infinity: the approximation of the first step is the exact value */
  const uint32_t specials[] = {0x00000000u, 0x80000000u, 0x7F800000u};
  for (unsigned i = 0; i < 3; ++i) {
    bad += to_bits(corrected(from_bits(specials[i]), from_bits(specials[i]))) != specials[i];
    ++cases;
  }
  printf("%llu %llu\n", bad, cases);
  return bad != 0;
}
