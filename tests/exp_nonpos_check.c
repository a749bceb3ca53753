/* Host-side check of the verification kernels' double-precision exponential (csrc/exp_nonpos.h) against the
 * long-double library routine, on a fixed grid.  Built and run by tests/test_exp_nonpos.py; prints the worst errors.
 *
 * Grid: three low-discrepancy sweeps x = -R frac(i phi), R = 2, 40, 745 (4e6 points each), the points next to every
 * multiple of ln2/64 down to -45 (where the argument reduction switches table entries), and a list of special
 * arguments.  Errors are in units of the last place of the exact result. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include "exp_nonpos.h"

static const double tab[64] = {DSBD_EXP2_TABLE_64};
static double worst_normal = 0.0, worst_normal_x = 0.0, worst_denormal = 0.0, worst_denormal_x = 0.0;
static long n_points = 0, n_monotone_violations = 0;

static void check(double x) {
  const double a = dsbd_exp_nonpos(x, tab);
  const long double b = expl((long double)x);
  ++n_points;
  if (b >= 2.2250738585072014e-308L) {
    const double bd = (double)b;
    const double ulp = nextafter(bd, INFINITY) - bd;
    const double e = fabs((double)(((long double)a - b) / (long double)ulp));
    if (e > worst_normal) { worst_normal = e; worst_normal_x = x; }
  } else {
    const double e = fabs((double)(((long double)a - b) / 4.9406564584124654e-324L));
    if (e > worst_denormal) { worst_denormal = e; worst_denormal_x = x; }
  }
}

int main(void) {
  const double phi = 0.6180339887498949;
  const double ranges[3] = {2.0, 40.0, 745.0};
  for (int r = 0; r < 3; ++r)
    for (long i = 1; i <= 4000000; ++i) {
      double f = (double)i * phi;
      f -= floor(f);
      check(-ranges[r] * f);
    }
  /* around the switching points of the reduction: k ln2/64 and the midpoints (k + 1/2) ln2/64 */
  for (int k = 0; k <= 2 * 64 * 65; ++k) {
    double x = -(double)k * 0.5 * 0.010830424696249145;
    for (int s = 0; s < 5; ++s) { check(x); x = nextafter(x, -INFINITY); }
    x = -(double)k * 0.5 * 0.010830424696249145;
    for (int s = 0; s < 5; ++s) { x = nextafter(x, 0.0); if (x <= 0.0) check(x); }
  }
  const double special[] = {0.0, -0.0, -1e-300, -4.9e-324, -1e-17, -0x1p-53, -0.5, -1.0, -0.6931471805599453, -87.3, -88.8,
                            -103.0, -700.0, -708.0, -708.3964185322641, -708.5, -709.78, -744.0, -745.0, -745.13, -745.2,
                            -800.0, -1000.0, -1001.0, -1e6, -1e300};
  for (unsigned i = 0; i < sizeof(special) / sizeof(special[0]); ++i) check(special[i]);
  /* never above 1, exactly 1 at 0, zero far down, and monotone over a fine sweep */
  double prev = dsbd_exp_nonpos(-50.0, tab);
  for (long i = 1; i <= 2000000; ++i) {
    const double x = -50.0 + 50.0 * (double)i / 2000000.0;
    const double v = dsbd_exp_nonpos(x, tab);
    if (v < prev) ++n_monotone_violations;
    prev = v;
  }
  printf("points %ld\n", n_points);
  printf("worst_normal_ulp %.4f at %.17g\n", worst_normal, worst_normal_x);
  printf("worst_denormal_ulp %.4f at %.17g\n", worst_denormal, worst_denormal_x);
  printf("exp0 %.17g\n", dsbd_exp_nonpos(0.0, tab));
  printf("exp_minus_1e6 %.17g\n", dsbd_exp_nonpos(-1e6, tab));
  printf("monotone_violations %ld\n", n_monotone_violations);
  return 0;
}
