/* Value-domain definition of round-to-nearest, ties-to-even, onto a binary
 * floating-point format with P significand bits (hidden bit included), smallest
 * normal exponent EMIN and largest exponent EMAX: among the two representable
 * neighbours of |x| pick the closer one; at equal distance pick the one whose
 * integer significand is even; beyond the largest finite value plus half a
 * spacing the result is infinity.  Nothing here touches bit patterns of the
 * 16-bit formats: it is used to check an encoder that does. */
#include <math.h>
#include <stdint.h>

static double nearest_value(double ax, int P, int emin, int emax) {
  if (ax == 0.0) return 0.0;
  int e;
  (void)frexp(ax, &e);
  e -= 1;                                   /* ax = f * 2^e, 1 <= f < 2 */
  if (e < emin) e = emin;                   /* subnormal range shares one spacing */
  double q = ldexp(1.0, e - (P - 1));       /* spacing of representable values near ax */
  double k = floor(ax / q);                 /* exact: division by a power of two */
  double lo = k * q, hi = (k + 1.0) * q;
  double dlo = ax - lo, dhi = hi - ax;      /* exact: binary32 input, coarser grid */
  double r;
  if (dlo < dhi) r = lo;
  else if (dhi < dlo) r = hi;
  else r = (fmod(k, 2.0) == 0.0) ? lo : hi;
  double maxv = ldexp(2.0 - ldexp(1.0, -(P - 1)), emax);
  if (r > maxv) r = INFINITY;
  return r;
}

/* x[i]: inputs; back[i]: decode(encode(x[i])) as produced by the code under test.
 * Returns the number of disagreements with the definition above. */
uint64_t pin_count_mismatch(const float* x, const float* back, uint64_t n, int dtype) {
  const int P = dtype == 0 ? 8 : 11, emin = dtype == 0 ? -126 : -14, emax = dtype == 0 ? 127 : 15;
  uint64_t bad = 0;
  for (uint64_t i = 0; i < n; ++i) {
    float xi = x[i], bi = back[i];
    if (isnan(xi)) { bad += !isnan(bi); continue; }
    if (isinf(xi)) { bad += !(isinf(bi) && (signbit(xi) == signbit(bi))); continue; }
    double want = nearest_value(fabs((double)xi), P, emin, emax);
    if (signbit(xi)) want = -want;
    bad += !((double)bi == want && signbit(bi) == signbit(xi));
  }
  return bad;
}
