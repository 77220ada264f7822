// Host check of exp64.h against libm: prints the largest error in ulps over a grid of arguments.
#include <cmath>
#include <cstdio>
#include <cstdint>
#include <cstring>
#include "exp64.h"

static double ulp_of(double v) {
  int e;
  std::frexp(v, &e);
  return std::ldexp(1.0, e - 53);
}

int main() {
  double worst = 0.0;
  uint64_t s = 0x9E3779B97F4A7C15ull;
  for (int i = 0; i < 4000000; ++i) {
    s ^= s << 13; s ^= s >> 7; s ^= s << 17;
    const double u = double(s >> 11) * (1.0 / 9007199254740992.0);
    // mostly (-60, 0], some down to -740 and a few small positive ones
    double x = (i % 8 == 0) ? -740.0 * u : ((i % 8 == 1) ? 5.0 * u : -60.0 * u);
    if (i % 16 == 2) x = double(float(x));                     // fp32-valued arguments, as in the kernels
    const long double want = expl((long double)x);
    const double got = tslt::exp64(x);
    if (want > 1e-290L) {
      const double err = std::fabs(double((long double)got - want)) / ulp_of(double(want));
      if (err > worst) worst = err;
    }
  }
  const bool edge = tslt::exp64(0.0) == 1.0 && tslt::exp64(-1e30) == 0.0 && tslt::exp64(-INFINITY) == 0.0 &&
                    tslt::exp64(-900.0) == 0.0;
  std::printf("max_ulp %.4f edge %d\n", worst, edge ? 1 : 0);
  return 0;
}
