// exp(x) in fp64 for the inverse-CDF passes, where x = s - s_max <= 0 (small positive arguments work
// too).  Range reduction x = n*ln2 + r with |r| <= ln2/2, a degree-13 Taylor polynomial for exp(r)
// (truncation error below 2^-57) and a scaling by 2^n; the result is within about one ulp of the
// correctly rounded value.  Arguments below -800 (including -inf) give exactly 0.  Branch-free, so
// that the compiler can interleave several evaluations.
#pragma once

#if defined(__HIPCC__)
#define TSLT_HD __host__ __device__ __forceinline__
#else
#define TSLT_HD inline
#endif

namespace tslt {

TSLT_HD double exp64(double x) {
  x = x > -800.0 ? x : -800.0;                                   // also maps -inf (and NaN) to -800
  const double n = __builtin_rint(x * 1.44269504088896338700e+00);
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
  return __builtin_ldexp(p, int(n));
}

}  // namespace tslt
