// Element-wise arithmetic of Ozaki scheme II in FP64 operations whose results are exact by construction.
// Every function is __host__ __device__: the kernels use them, and the same source compiled for the host
// backs the unit tests of the exactness arguments written next to each step.
#ifndef OZ2_MATH_H
#define OZ2_MATH_H

#include <hip/hip_runtime.h>
#include <math.h>

#include "oz2_internal.h"

#define OZ2_HD __host__ __device__ __forceinline__

// ---------------------------------------------------------------------------------------------------
// Algorithm 1 lines 2-5 for one element.
//   x = trunc(a * 2^shift) is an integer-valued double (|x| < 2^kappa, possibly far above 2^53: its low
//   bits are zero then).  Split x = x2*2^64 + x1*2^32 + x0 with integer parts of the same sign
//   (|x1|,|x0| < 2^32); then  y_t = x2*c64_t + x1*c32_t + x0  is congruent to x modulo p_t, exact in
//   FP64 and below 2^51 in magnitude, so one rounded quotient gives the symmetric residue exactly:
//   |y/p * 2^-52| < 1/(2p) is the distance of y/p from the nearest rounding tie for odd p.  For
//   p = 256 a tie can occur and yields +128, which wraps to -128 in INT8 (Section 3.1).
// ---------------------------------------------------------------------------------------------------
struct Oz2Split {
  double x2, x1, x0;
};

template <bool TWO_LEVEL>
OZ2_HD Oz2Split oz2_scale_trunc_split(double a, int shift) {
  Oz2Split s;
  double x = trunc(ldexp(a, shift));
  if (TWO_LEVEL) {
    s.x2 = trunc(x * 0x1p-64);
    double rem = fma(-s.x2, 0x1p64, x);
    s.x1 = trunc(rem * 0x1p-32);
    s.x0 = fma(-s.x1, 0x1p32, rem);
  } else {
    s.x2 = 0.0;
    s.x1 = trunc(x * 0x1p-32);
    s.x0 = fma(-s.x1, 0x1p32, x);
  }
  return s;
}

template <bool TWO_LEVEL>
OZ2_HD int oz2_sym_residue(const Oz2Split& s, double p, double inv_p, double c32, double c64) {
  double y = fma(s.x1, c32, s.x0);
  if (TWO_LEVEL) y = fma(s.x2, c64, y);
  double q = rint(y * inv_p);
  double r = fma(-q, p, y);
  return (int)r;
}

// ---------------------------------------------------------------------------------------------------
// Section 4.1, INT8-product bound: ceil(|a| 2^sh) with sh = 5 - floor(log2 of the vector's maximum), an
// integer in [0, 64] that bounds |a| 2^sh from above.  The scaling is exact unless it underflows to zero,
// and the ceiling of any positive value is at least one.
// ---------------------------------------------------------------------------------------------------
OZ2_HD int oz2_bound6(double a, int sh) {
  double q = ceil(ldexp(fabs(a), sh));
  if (a != 0.0 && q == 0.0) q = 1.0;
  return (int)q;
}

// ---------------------------------------------------------------------------------------------------
// Algorithm 1 line 7: c'' = c' - floor(c'/p) p for an INT32 c', as a double in [0, p).
//   floor((c' + 1/2)/p) == floor(c'/p) and (c' + 1/2)/p stays 1/(2p) away from every integer, far more
//   than the rounding error 2^31/p * 2^-52 of the fused multiply-add, so the floor is exact.
// ---------------------------------------------------------------------------------------------------
OZ2_HD double oz2_floor_mod(int c, double p, double inv_p, double half_inv_p) {
  double x = (double)c;
  double q = floor(fma(x, inv_p, half_inv_p));
  return fma(-q, p, x);
}

// ---------------------------------------------------------------------------------------------------
// Algorithm 1 lines 8-10 and the rounding of line 11.
//   Input: S[l] = sum_t c''_t * w_{t,l} (integers below 2^53, exact), i.e. Y = sum_l S[l] 2^(40 l).
//   Output: the double nearest to X = Y mod M (symmetric, Section 2.1) as r * 2^e2.
//   Steps: Q = rint(Y/M) from a floating estimate; T[l] = S[l] - Q*m_l exactly; if the estimate is too
//   close to a half-integer to trust Q, X is compared with M/2 exactly on its digits; carries are
//   propagated so that X = sum_l D[l] 2^(40 l) with |D[l]| <= 2^39 below the top digit; the top three
//   nonzero-led digits are rounded once with the remaining digits acting as a sticky term.
// ---------------------------------------------------------------------------------------------------
template <int L>
OZ2_HD void oz2_carry(double* T) {
#pragma unroll
  for (int l = 0; l + 1 < L; ++l) {
    double c = rint(T[l] * 0x1p-40);
    T[l] = fma(-c, 0x1p40, T[l]);
    T[l + 1] += c;
  }
}

// ---------------------------------------------------------------------------------------------------
// Digit route to the same S[l] (matrix-core CRT kernel): D[i] = sum_t c''_t dig[i][t] for the sixteen balanced
// base-256 digits of the weights in the symmetric range, |D[i]| <= 16 * 255 * 128 < 2^20, so that
//   Y' = sum_i D[i] 256^i  is congruent to  Y = sum_t c''_t W_t  modulo M,  |Y'| <= 2^11 M.
// Limb l collects the digits 5 l .. 5 l + 4 (the top limb all that remain): integers below 2^53, exact.  In a
// top limb with few digits in use the upper D[i] are zero (|Ws| <= M/2 < 2^(40 L - 1)).
// ---------------------------------------------------------------------------------------------------
template <int L>
OZ2_HD void oz2_digits_to_limbs(const int* D, const double* start, double* S) {
#pragma unroll
  for (int l = 0; l < L; ++l) {
    const int first = 5 * l, last = l + 1 < L ? 5 * l + 4 : 15;
    double v = (double)D[last];
#pragma unroll
    for (int i = last - 1; i >= first; --i) v = fma(v, 256.0, (double)D[i]);
    S[l] = v + start[l];  // the digit sums were formed on c'' - 128: start holds 128 sum_t dig in limb form
  }
}

template <int L>
OZ2_HD double oz2_crt_reduce(const double* S, const Oz2CrtConsts& cc, int* e2) {
  double yest = 0.0;
#pragma unroll
  for (int l = L - 1; l >= 0; --l) yest = fma(S[l], cc.rinv[l], yest);
  double Q = rint(yest);
  double frac = yest - Q;

  constexpr int LP = L < 3 ? 3 : L;
  double D[LP];
#pragma unroll
  for (int l = 0; l < LP; ++l) D[l] = l < L ? fma(-Q, cc.mlimb[l], S[l]) : 0.0;

  if (fabs(frac) > 0.4999990463256836) {  // 0.5 - 2^-20: the estimate (error < 2^-36) cannot decide
    double sgn = frac > 0.0 ? 1.0 : -1.0;
    double U[L];
#pragma unroll
    for (int l = 0; l < L; ++l) U[l] = sgn * D[l] - cc.mhalf[l];
    oz2_carry<L>(U);
    double lead = 0.0;  // highest nonzero digit of sgn*X - M/2
#pragma unroll
    for (int l = 0; l < L; ++l)
      if (U[l] != 0.0) lead = U[l];
    if (lead > 0.0 || (lead == 0.0 && sgn > 0.0)) {  // X outside [-M/2, M/2)
      Q += sgn;
#pragma unroll
      for (int l = 0; l < L; ++l) D[l] = fma(-Q, cc.mlimb[l], S[l]);
    }
  }
  oz2_carry<L>(D);

  // window of three digits led by the highest nonzero one (or the lowest three)
  double dh = D[2], dm = D[1], dl = D[0], rest = 0.0;
  int shift = 0;
#pragma unroll
  for (int w = 3; w < LP; ++w) {
    if (D[w] != 0.0) {
      dh = D[w];
      dm = D[w - 1];
      dl = D[w - 2];
      double rr = 0.0;
#pragma unroll
      for (int i = 0; i <= w - 3; ++i)
        if (D[i] != 0.0) rr = D[i];
      rest = rr;
      shift = OZ2_LIMB_BITS * (w - 2);
    }
  }
  // the digits below the window only matter through their sign: move dl by a quarter unit
  double lo = dl + (rest > 0.0 ? 0.25 : (rest < 0.0 ? -0.25 : 0.0));
  double hi = dh * 0x1p80, mid = dm * 0x1p40;
  double a = hi + mid;          // |hi| >= 2^80 > |mid| or hi == 0: Fast2Sum is exact
  double b = mid - (a - hi);
  double tail;
  if (b != 0.0) {
    // |b| >= 2^40 > 2|lo|: lo can only break an exact tie of a + b; nudge b by one part in 2^52
    tail = lo != 0.0 ? fma(fabs(b), copysign(0x1p-52, lo), b) : b;
  } else {
    tail = lo;
  }
  *e2 = shift;
  return a + tail;
}

#endif
