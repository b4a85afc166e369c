/* CPU check of the fused QAT kernel's square root of a corrected second moment, sqrt(v / c) for a bf16 v and a
 * launch-uniform c in [2^-20, 1], read from two tables:
 *     E = exponent field of v = 2 H + p,  f = its 7 significand bits
 *     roots[p, f] = RN(sqrt(RN((1.f 2^(p+1)) / c)))          256 entries
 *     scales[H]   = 0 for H = 0;  2^(H - 64) for 1 <= H <= 116;  NaN above
 *     result      = roots[p, f] * scales[H]
 * Claim: wherever the result is not a NaN it is RN(sqrt(RN(v / c))) bit for bit (both correctly rounded operations
 * commute with the scaling by (2^(H-64))^2 while every value stays normal), except for H = 0 (v < 2^-125), where it
 * is zero and the true root is below 2^-52 (the kernel adds an eps of at least 2^-28, whose sum with such a root is
 * eps itself).  Checked for every non-negative bf16 code against `count` values of c (ends of the range, all-ones
 * and all-zeros significands, random ones).  Prints: counterexamples, cases tried. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float from_bits(uint32_t u) { float v; memcpy(&v, &u, 4); return v; }
static uint32_t to_bits(float v) { uint32_t u; memcpy(&u, &v, 4); return u; }

int main(int argc, char** argv) {
  const int count = argc > 1 ? atoi(argv[1]) : 300;
  uint64_t state = 0x2545F4914F6CDD1Dull, bad = 0, cases = 0;
  for (int it = 0; it < count; ++it) {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    const int e = -20 + (int)(state % 21);
    uint32_t m = (uint32_t)(state >> 20) & 0x7FFFFFu;
    if (it % 7 == 0) m = 0;
    if (it % 7 == 1) m = 0x7FFFFFu;
    if (it % 11 == 0) m &= 0x7F0000u;
    volatile float c = from_bits(((uint32_t)(e + 127) << 23) | m);
    if (c > 1.0f || it == 2) c = 1.0f;
    if (it == 3) c = 0x1p-20f;
    float roots[256], scales[128];
    for (uint32_t i = 0; i < 256; ++i) {
      volatile float x = from_bits(((128u + (i >> 7)) << 23) | ((i & 127u) << 16));
      volatile float y = x / c;
      roots[i] = sqrtf(y);
    }
    for (uint32_t h = 0; h < 128; ++h) scales[h] = h == 0 ? 0.0f : (h <= 116 ? from_bits((h + 63u) << 23) : NAN);
    for (uint32_t code = 0; code < 0x8000u; ++code) {
      const uint32_t bits = code << 16;
      volatile float v = from_bits(bits);
      volatile float q = v / c;
      const float want = sqrtf(q);
      const float got = roots[(bits >> 16) & 0xFFu] * scales[bits >> 24];
      ++cases;
      if (isnan(got)) continue;   /* the wave recomputes */
      if ((bits >> 24) == 0) bad += !(got == 0.0f && want < 0x1p-52f);
      else bad += to_bits(got) != to_bits(want);
    }
  }
  printf("%llu %llu\n", (unsigned long long)bad, (unsigned long long)cases);
  return bad != 0;
}
