// Host check of the two division shortcuts the quantizer kernel relies on (IEEE fp32, fma as one
// rounding -- the same arithmetic the GPU instructions perform):
//  (1) scale: d / qmax for qmax 3 and 15 equals  q0 = d * c,  q = fma(fma(-qmax, q0, d), c, q0)  with
//      c = fl(1 / qmax), for every fp32 d in [2^-26, 2^18] (every difference of two finite fp16 values
//      lies there, or is 0);
//  (2) codes: for every positive finite fp16 scale s, one Newton step on a reciprocal seed up to 2 ulps
//      off gives y = RN(1 / s), and  q0 = d * y,  q = fma(fma(-s, q0, d), y, q0)  equals d / s for
//      numerators d on and within 4 ulps of every half-integer multiple of s up to 1.5 * qmax + 1.5
//      (where rounding to a code is decided) and for random ones.
// Prints one line per part; exit status 0 iff no mismatch.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float from_bits(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float half_value(uint16_t h) {  // positive finite fp16 bit pattern
  const int e = (h >> 10) & 31, m = h & 1023;
  return e == 0 ? ldexpf((float)m, -24) : ldexpf((float)(m + 1024), e - 25);
}
static float quotient(float d, float s) { volatile float q = d / s; return q; }

int main(void) {
  long bad = 0;
  const float qmaxes[2] = {3.0f, 15.0f};
  for (int k = 0; k < 2; ++k) {
    const float b = qmaxes[k], c = quotient(1.0f, b);
    long n = 0, miss = 0;
    for (uint32_t u = to_bits(0x1p-26f); u <= to_bits(0x1p18f); ++u, ++n) {
      const float d = from_bits(u), q0 = d * c;
      if (fmaf(fmaf(-b, q0, d), c, q0) != quotient(d, b)) ++miss;
    }
    printf("scale division by %g: %ld numerators, %ld mismatches\n", b, n, miss);
    bad += miss;
  }
  long nq = 0, miss_y = 0, miss_q = 0;
  srand(1);
  for (uint32_t hb = 1; hb < 0x7c00; ++hb) {
    const float s = half_value((uint16_t)hb), y = quotient(1.0f, s);
    for (int k = -2; k <= 2; ++k) {
      const float y0 = from_bits(to_bits(y) + k);
      if (fmaf(fmaf(-s, y0, 1.0f), y0, y0) != y) ++miss_y;
    }
    for (int qi = 0; qi < 2; ++qi) {
      const int qmax = (int)qmaxes[qi];
      for (int j = 0; j <= 3 * qmax + 3; ++j)
        for (int k = -4; k <= 4; ++k) {
          const float d = from_bits(to_bits(0.5f * j * s) + k);
          if (!(d >= 0.0f) || (d != 0.0f && d < 0x1p-24f)) continue;   // numerators are multiples of 2^-24
          const float q0 = d * y;
          ++nq;
          if (fmaf(fmaf(-s, q0, d), y, q0) != quotient(d, s)) ++miss_q;
        }
      for (int t = 0; t < 200; ++t) {
        const float d = s * (1.5f * qmax + 1.0f) * ((float)rand() / (float)RAND_MAX), q0 = d * y;
        ++nq;
        if (fmaf(fmaf(-s, q0, d), y, q0) != quotient(d, s)) ++miss_q;
      }
    }
  }
  printf("reciprocal refinement: %ld mismatches; code quotients: %ld cases, %ld mismatches\n", miss_y, nq, miss_q);
  bad += miss_y + miss_q;
  return bad ? 1 : 0;
}
