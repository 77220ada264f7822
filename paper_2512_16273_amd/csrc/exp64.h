// exp(x) in fp64 for the inverse-CDF passes, where x = s - s_max <= 0 (small positive arguments work
// too).  Range reduction x = n*ln2 + r with |r| <= ln2/2, a degree-13 Taylor polynomial for exp(r)
// (truncation error below 2^-57) and a scaling by 2^n; the result is within about one ulp of the
// correctly rounded value.  Arguments below about -709 (including -inf and NaN) give exactly 0:
// results that would be subnormal are flushed.  Branch-free, and written with the operations that
// run at full rate on gfx950: rounding to an integer and the scaling are done with a "magic number"
// addition and an exponent-field construction instead of rint / convert / ldexp, which issue at a
// quarter of the rate there.
#pragma once
#include <stdint.h>
#include <string.h>

#if defined(__HIPCC__)
#define TSLT_HD __host__ __device__ __forceinline__
#else
#define TSLT_HD inline
#endif

namespace tslt {

TSLT_HD double exp64(double x) {
  x = x > -800.0 ? x : -800.0;                                   // also maps -inf (and NaN) to -800
  // n = round(x / ln2): adding 1.5 * 2^52 leaves n in the low mantissa bits of t
  const double kMagic = 6755399441055744.0;
  const double t = __builtin_fma(x, 1.44269504088896338700e+00, kMagic);
  const double n = t - kMagic;
  uint64_t tb;
  memcpy(&tb, &t, 8);
  int32_t ni = int32_t(uint32_t(tb));                             // n as an integer (|n| < 2^31)
  double r = __builtin_fma(n, -6.93147180369123816490e-01, x);   // high part of ln2 (low 32 bits zero)
  r = __builtin_fma(n, -1.90821492927058770002e-10, r);          // low part of ln2
  double p = 1.6059043836821613e-10;                              // 1/13!
  p = __builtin_fma(p, r, 2.08767569878681e-09);                  // 1/12!
  p = __builtin_fma(p, r, 2.505210838544172e-08);                 // 1/11!
  p = __builtin_fma(p, r, 2.755731922398589e-07);                 // 1/10!
  p = __builtin_fma(p, r, 2.7557319223985893e-06);                // 1/9!
  p = __builtin_fma(p, r, 2.48015873015873e-05);                  // 1/8!
  p = __builtin_fma(p, r, 1.984126984126984e-04);                 // 1/7!
  p = __builtin_fma(p, r, 1.388888888888889e-03);                 // 1/6!
  p = __builtin_fma(p, r, 8.333333333333333e-03);                 // 1/5!
  p = __builtin_fma(p, r, 4.1666666666666664e-02);                // 1/4!
  p = __builtin_fma(p, r, 1.6666666666666666e-01);                // 1/3!
  p = __builtin_fma(p, r, 0.5);
  p = __builtin_fma(p, r, 1.0);
  p = __builtin_fma(p, r, 1.0);
  // 2^n built in the exponent field; n <= -1023 gives the bit pattern of 0.0
  ni = ni > -1023 ? ni : -1023;
  const uint64_t sb = uint64_t(uint32_t(ni + 1023)) << 52;
  double scale;
  memcpy(&scale, &sb, 8);
  return p * scale;
}

}  // namespace tslt
