// fp64 exponential for non-positive arguments, shared by the sampling acceptance kernels: internal
// to the library. gfx950 (CDNA4) only.
#ifndef FSPAD_EXP_NONPOS_H
#define FSPAD_EXP_NONPOS_H

#include <hip/hip_runtime.h>

namespace fspad_detail {

// exp(x) for x <= 0 in fp64: x = n ln2 + r, |r| <= ln2/2, degree-11 Taylor polynomial
// (truncation below 1e-14 relative), scaled by 2^n. n is rounded with the 1.5*2^52 shift (its
// integer value then sits in the low word of the shifted number) and 2^n is assembled from its
// exponent bits, which keeps the whole routine on full-rate multiply-adds. Returns 0 below
// -708 (where the true value is under 1e-307: its absence moves no sum by a representable amount).
__device__ __forceinline__ double exp_nonpos(double x) {
  // Branch-free on purpose: with an early return every call becomes a block of its own and the
  // compiler rebuilds the 64-bit constants in each (more moves than arithmetic).
  const bool vanishes = !(x >= -708.0);  // also catches NaN
  x = fmax(x, -708.0);                   // NaN -> -708: the arithmetic below stays in range
  const double shift = 6755399441055744.0;  // 1.5 * 2^52
  const double t = fma(x, 1.4426950408889634074, shift);
  const double n = t - shift;
  const int ni = (int)__double2loint(t);   // low word of the shifted value: n as a 32-bit integer (n in [-1022, 0])
  double r = fma(-n, 6.93147180369123816490e-01, x);
  r = fma(-n, 1.90821492927058770002e-10, r);
  double p = 1.0 / 39916800.0;
  p = fma(p, r, 1.0 / 3628800.0);
  p = fma(p, r, 1.0 / 362880.0);
  p = fma(p, r, 1.0 / 40320.0);
  p = fma(p, r, 1.0 / 5040.0);
  p = fma(p, r, 1.0 / 720.0);
  p = fma(p, r, 1.0 / 120.0);
  p = fma(p, r, 1.0 / 24.0);
  p = fma(p, r, 1.0 / 6.0);
  p = fma(p, r, 0.5);
  p = fma(p, r, 1.0);
  p = fma(p, r, 1.0);
  const double scale = __hiloint2double((ni + 1023) << 20, 0);   // 2^n
  return vanishes ? 0.0 : p * scale;
}

}  // namespace fspad_detail
#endif
