// Host-side check of the quotient the activation quantiser kernel computes (csrc/fq_quantize.hip):
// for every finite bf16 absmax > 0 (every STRIDE-th one; STRIDE = 1 is the exhaustive run) with
// s = absmax / 448 in [2^-60, 2^60], and every finite bf16 x with |x| <= absmax, the E4M3 code of
//     copysign(fma(fma(-q, s, x), r, q), x),  q = x * r,  r = 1 / s        (all FP32, IEEE)
// must equal the E4M3 code of the IEEE quotient x / s.  Exit status 0 = no difference.
// usage: fast_quotient_check [STRIDE]
#include <stdio.h>
#include <stdint.h>
#include <string.h>
#include <math.h>
#include <omp.h>
static inline float bf(uint32_t b) { uint32_t u = b << 16; float f; memcpy(&f, &u, 4); return f; }
static inline uint32_t bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
// E4M3 (OCP, bias 7) round-to-nearest-even of a float with |f| <= 448
static uint8_t e4m3(float f) {
  uint32_t u = bits(f), sign = (u >> 24) & 0x80;
  float a = fabsf(f);
  if (a == 0.f) return (uint8_t)sign;
  int e; float m = frexpf(a, &e);            // a = m * 2^e, m in [0.5, 1)
  int ex = e - 1;                             // a = (2m) * 2^ex, 2m in [1, 2)
  if (ex < -6) {                              // subnormal range: units of 2^-9
    float q = a * 512.0f; float rq = nearbyintf(q);   // RNE (default rounding mode)
    int k = (int)rq; if (k >= 8) return (uint8_t)(sign | 0x08);
    return (uint8_t)(sign | k);
  }
  float frac = (2.0f * m - 1.0f) * 8.0f;      // in [0, 8)
  int k = (int)nearbyintf(frac);
  if (k == 8) { k = 0; ex += 1; }
  int code = ((ex + 7) << 3) | k;
  if (code > 0x7E) code = 0x7E;
  return (uint8_t)(sign | code);
}
static inline float clampf(float v) { return fminf(fmaxf(v, -448.f), 448.f); }
#include <stdlib.h>
int main(int argc, char** argv) {
  const int stride = argc > 1 ? atoi(argv[1]) : 1;
  long long bad = 0, total = 0, bitdiff = 0;
  #pragma omp parallel for schedule(dynamic, 16) reduction(+:bad,total,bitdiff)
  for (int ab = 1; ab < 0x7F80; ab += stride) {
    volatile float amax = bf(ab);
    float s = amax / 448.0f;
    if (!(s >= 0x1p-60f && s <= 0x1p60f)) continue;
    float r = 1.0f / s;
    for (int xb = 0; xb <= ab; ++xb) {
      for (int sg = 0; sg < 2; ++sg) {
        float x = bf(xb | (sg << 15));
        float want = x / s;
        float q = x * r;
        float e = fmaf(-q, s, x);
        float got = copysignf(fmaf(e, r, q), x);
        ++total;
        if (bits(want) != bits(got)) ++bitdiff;
        if (e4m3(clampf(want)) != e4m3(clampf(got))) { ++bad; if (bad < 5) printf("CODE diff amax=%a x=%a want=%a got=%a\n", amax, x, want, got); }
      }
    }
  }
  printf("total %lld  quotient bit differences %lld  E4M3 code differences %lld\n", total, bitdiff, bad);
  return bad != 0;
}
