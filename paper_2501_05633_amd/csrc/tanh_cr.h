// tanh (and, further down, erf) of a non-negative binary32 argument, rounded
// correctly to binary32.
//
// The selection score needs tanh to be the same function on every machine, so
// it is defined as the correctly rounded value and computed here from IEEE
// binary64 +, -, *, /, fma only (no device math library):
//
//   tanh(x) = E / (E + 2),  E = expm1(2x),  2x = n ln2 + r,  |r| <= ln2/2,
//   expm1(r) by its Taylor series (degree 14; the remainder is below 2^-60 of
//   the sum), E = 2^n expm1(r) + (2^n - 1).
//
// The binary64 result carries a relative error below 2^-49; when rounding it
// to binary32 could depend on that error (the value lies within 2^-47 of a
// rounding boundary) the same evaluation is repeated in double-double
// arithmetic (about 100 bits), which settles it.
#pragma once
#include <hip/hip_runtime.h>

namespace rtk {

struct dd { double hi, lo; };

__device__ __forceinline__ dd dd_two_sum(double a, double b) {
  double s = a + b;
  double bb = s - a;
  double err = (a - (s - bb)) + (b - bb);
  return {s, err};
}
__device__ __forceinline__ dd dd_quick_two_sum(double a, double b) {  // |a| >= |b|
  double s = a + b;
  return {s, b - (s - a)};
}
__device__ __forceinline__ dd dd_two_prod(double a, double b) {
  double p = a * b;
  return {p, __fma_rn(a, b, -p)};
}
__device__ __forceinline__ dd dd_add(dd a, dd b) {
  dd s = dd_two_sum(a.hi, b.hi);
  dd t = dd_two_sum(a.lo, b.lo);
  s.lo += t.hi;
  s = dd_quick_two_sum(s.hi, s.lo);
  s.lo += t.lo;
  return dd_quick_two_sum(s.hi, s.lo);
}
__device__ __forceinline__ dd dd_add_d(dd a, double b) {
  dd s = dd_two_sum(a.hi, b);
  s.lo += a.lo;
  return dd_quick_two_sum(s.hi, s.lo);
}
__device__ __forceinline__ dd dd_mul(dd a, dd b) {
  dd p = dd_two_prod(a.hi, b.hi);
  p.lo += a.hi * b.lo + a.lo * b.hi;
  return dd_quick_two_sum(p.hi, p.lo);
}
__device__ __forceinline__ dd dd_mul_d(dd a, double b) {
  dd p = dd_two_prod(a.hi, b);
  p.lo += a.lo * b;
  return dd_quick_two_sum(p.hi, p.lo);
}
__device__ __forceinline__ dd dd_div(dd a, dd b) {
  double q1 = a.hi / b.hi;
  dd r = dd_add(a, dd_mul_d(b, -q1));
  double q2 = r.hi / b.hi;
  r = dd_add(r, dd_mul_d(b, -q2));
  double q3 = r.hi / b.hi;
  dd q = dd_quick_two_sum(q1, q2);
  return dd_add_d(q, q3);
}

// ln 2 split into three binary64 pieces (each the rounding of what is left).
#define RTK_LN2_A 0x1.62e42fefa39efp-1
#define RTK_LN2_B 0x1.abc9e3b39803fp-56
#define RTK_LN2_C 0x1.7b57a079a1934p-111
#define RTK_LOG2E 0x1.71547652b82fep+0

// One rounding of a positive double-double value hi + lo to binary32.
__device__ __forceinline__ float dd_round_f32(dd y) {
  float f = (float)y.hi;
  const double fl = (double)f;
  const double diff = (y.hi - fl) + y.lo;
  if (diff > 0.0) {
    float up = __uint_as_float(__float_as_uint(f) + 1u);
    if (diff > 0.5 * ((double)up - fl)) f = up;
  } else if (diff < 0.0) {
    float dn = __uint_as_float(__float_as_uint(f) - 1u);
    if (-diff > 0.5 * (fl - (double)dn)) f = dn;
  }
  return f;
}

// Slow, ~100-bit evaluation (only reached for arguments whose tanh lies
// extremely close to the midpoint of two binary32 numbers).
__device__ __noinline__ float tanh_f32_dd(float xf) {
  const double t = 2.0 * (double)xf;                       // exact
  const double n = rint(t * RTK_LOG2E);
  // r = t - n ln2 in double-double
  dd r = dd_two_prod(-n, RTK_LN2_A);
  r = dd_add_d(r, t);
  r = dd_add(r, dd_two_prod(-n, RTK_LN2_B));
  r = dd_add_d(r, -n * RTK_LN2_C);
  // expm1(r / 256) by its Taylor series in nested form
  //   expm1(s) = s (1 + s/2 (1 + s/3 (1 + ... (1 + s/12)))),
  // then 8 doublings  expm1(2u) = 2 expm1(u) + expm1(u)^2.
  dd s = {r.hi * 0.00390625, r.lo * 0.00390625};
  dd h = {1.0, 0.0};
  for (int kk = 12; kk >= 2; --kk) {
    dd kd = {(double)kk, 0.0};
    h = dd_add_d(dd_div(dd_mul(s, h), kd), 1.0);
  }
  dd q = dd_mul(s, h);
  for (int i = 0; i < 8; ++i) {
    dd q2 = dd_mul(q, q);
    q = dd_add(dd_mul_d(q, 2.0), q2);
  }
  // E = 2^n q + (2^n - 1),  tanh = E / (E + 2)
  const double sc = ldexp(1.0, (int)n);
  dd E = dd_add_d(dd_mul_d(q, sc), sc - 1.0);
  dd y = dd_div(E, dd_add_d(E, 2.0));
  return dd_round_f32(y);
}

__device__ __forceinline__ float tanh_f32_cr(float xf) {
  if (!(xf < 9.02f)) return 1.0f;          // tanh(x) >= 1 - 2^-25 from x = 9.011 on
  const double t = 2.0 * (double)xf;       // exact
  const double n = rint(t * RTK_LOG2E);
  double r = __fma_rn(-n, RTK_LN2_A, t);
  r = __fma_rn(-n, RTK_LN2_B, r);
  double p = 1.0 / 87178291200.0;                       // 1/14!
  p = __fma_rn(p, r, 1.0 / 6227020800.0);               // 1/13!
  p = __fma_rn(p, r, 1.0 / 479001600.0);
  p = __fma_rn(p, r, 1.0 / 39916800.0);
  p = __fma_rn(p, r, 1.0 / 3628800.0);
  p = __fma_rn(p, r, 1.0 / 362880.0);
  p = __fma_rn(p, r, 1.0 / 40320.0);
  p = __fma_rn(p, r, 1.0 / 5040.0);
  p = __fma_rn(p, r, 1.0 / 720.0);
  p = __fma_rn(p, r, 1.0 / 120.0);
  p = __fma_rn(p, r, 1.0 / 24.0);
  p = __fma_rn(p, r, 1.0 / 6.0);
  p = __fma_rn(p, r, 0.5);
  const double q = __fma_rn(r * r, p, r);               // expm1(r)
  const double sc = ldexp(1.0, (int)n);
  const double E = __fma_rn(sc, q, sc - 1.0);           // expm1(2x)
  const double y = E / (E + 2.0);
  const float lo = (float)(y * (1.0 - 0x1p-47));
  const float hi = (float)(y * (1.0 + 0x1p-47));
  if (lo == hi) return lo;
  return tanh_f32_dd(xf);
}

// ------------------------------------------------------------------- erf ----
// erf of a non-negative binary32 argument, rounded correctly to binary32 (the
// likelihood of a Gaussian innovation).  From binary64 operations only:
//
//   erf(x) = (2/sqrt(pi)) exp(-x^2) sum_{n>=0} 2^n x^(2n+1) / (1*3*5*...*(2n+1)),
//
// a series of positive terms (no cancellation; at most 63 terms up to the
// saturation point), with exp(-x^2) from the same argument reduction and
// Taylor polynomial as above (x^2 is exact in binary64).  The binary64 result
// carries a relative error below 2^-45; when rounding it to binary32 could
// depend on that error the evaluation is repeated in double-double arithmetic.
#define RTK_2_SQRTPI_HI 0x1.20dd750429b6dp+0
#define RTK_2_SQRTPI_LO 0x1.1ae3a914fed80p-56

__device__ __noinline__ float erf_f32_dd(float xf) {
  const double x = (double)xf;
  const double t = -(x * x);                               // exact
  const double n = rint(t * RTK_LOG2E);
  dd r = dd_two_prod(-n, RTK_LN2_A);
  r = dd_add_d(r, t);
  r = dd_add(r, dd_two_prod(-n, RTK_LN2_B));
  r = dd_add_d(r, -n * RTK_LN2_C);
  dd s = {r.hi * 0.00390625, r.lo * 0.00390625};
  dd h = {1.0, 0.0};
  for (int kk = 12; kk >= 2; --kk) {
    dd kd = {(double)kk, 0.0};
    h = dd_add_d(dd_div(dd_mul(s, h), kd), 1.0);
  }
  dd q = dd_mul(s, h);
  for (int i = 0; i < 8; ++i) {
    dd q2 = dd_mul(q, q);
    q = dd_add(dd_mul_d(q, 2.0), q2);
  }
  const double sc = ldexp(1.0, (int)n);
  dd ex = dd_mul_d(dd_add_d(q, 1.0), sc);                  // exp(-x^2)
  const dd x2 = {2.0 * x * x, 0.0};                        // exact
  dd term = {x, 0.0}, sum = {x, 0.0};
  for (int kk = 1; kk < 160; ++kk) {                       // (about 100 terms at the saturation point)
    dd kd = {(double)(2 * kk + 1), 0.0};
    term = dd_div(dd_mul(term, x2), kd);
    sum = dd_add(sum, term);
    if (term.hi < sum.hi * 0x1p-100) break;
  }
  const dd c = {RTK_2_SQRTPI_HI, RTK_2_SQRTPI_LO};
  return dd_round_f32(dd_mul(dd_mul(c, ex), sum));
}

__device__ __forceinline__ float erf_f32_cr(float xf) {
  if (!(xf < 3.92f)) return 1.0f;          // erf(x) >= 1 - 2^-25 from x = 3.9193 on
  if (xf == 0.0f) return 0.0f;
  const double x = (double)xf;
  const double t = -(x * x);               // exact
  const double n = rint(t * RTK_LOG2E);
  double r = __fma_rn(-n, RTK_LN2_A, t);
  r = __fma_rn(-n, RTK_LN2_B, r);
  double p = 1.0 / 87178291200.0;                       // 1/14!
  p = __fma_rn(p, r, 1.0 / 6227020800.0);
  p = __fma_rn(p, r, 1.0 / 479001600.0);
  p = __fma_rn(p, r, 1.0 / 39916800.0);
  p = __fma_rn(p, r, 1.0 / 3628800.0);
  p = __fma_rn(p, r, 1.0 / 362880.0);
  p = __fma_rn(p, r, 1.0 / 40320.0);
  p = __fma_rn(p, r, 1.0 / 5040.0);
  p = __fma_rn(p, r, 1.0 / 720.0);
  p = __fma_rn(p, r, 1.0 / 120.0);
  p = __fma_rn(p, r, 1.0 / 24.0);
  p = __fma_rn(p, r, 1.0 / 6.0);
  p = __fma_rn(p, r, 0.5);
  const double q = __fma_rn(r * r, p, r);               // expm1(r)
  const double sc = ldexp(1.0, (int)n);
  const double ex = __fma_rn(sc, q, sc);                // exp(-x^2)
  const double x2 = 2.0 * x * x;
  double term = x, sum = x;
  for (int kk = 1; kk < 96; ++kk) {
    term = term * x2 / (double)(2 * kk + 1);
    sum += term;
    if (term < sum * 0x1p-60) break;
  }
  const double y = RTK_2_SQRTPI_HI * ex * sum;
  const float lo = (float)(y * (1.0 - 0x1p-43));
  const float hi = (float)(y * (1.0 + 0x1p-43));
  if (lo == hi) return lo;
  return erf_f32_dd(xf);
}

// ------------------------------------------------------------------- pow ----
// x^y for a non-negative binary32 x and a binary32 exponent 0 < y < 1, rounded
// correctly to binary32 (the prior |a|^y with a general exponent).  From
// binary64 operations only:
//
//   x = m 2^e with sqrt(1/2) <= m < sqrt(2),  ln m = 2 atanh(s), s = (m-1)/(m+1)
//   (|s| <= 0.1716: twelve terms of the odd series),  L = y (e ln2 + ln m),
//   x^y = exp(L) by the argument reduction and Taylor polynomial used above.
//
// |L| stays below 104, so the binary64 result carries a relative error below
// 2^-44; when rounding it to binary32 could depend on that error the evaluation
// is repeated in double-double arithmetic.
__device__ __forceinline__ void split_m_e(float xf, double* m, int* e) {
  // xf > 0, finite (denormals included): exact in binary64
  const double x = (double)xf;
  int ex;
  double mm = frexp(x, &ex);                 // x = mm 2^ex, 0.5 <= mm < 1
  if (mm < 0x1.6a09e667f3bcdp-1) { mm *= 2.0; ex -= 1; }
  *m = mm;
  *e = ex;
}

__device__ __noinline__ float pow_f32_dd(float xf, float yf) {
  double m; int e;
  split_m_e(xf, &m, &e);
  // s = (m - 1) / (m + 1) in double-double (m - 1 and m + 1 are exact sums of two doubles)
  const dd sn = dd_two_sum(m, -1.0), sd = dd_two_sum(m, 1.0);
  const dd sv = dd_div(sn, sd);
  const dd s2 = dd_mul(sv, sv);
  dd acc = {0.0, 0.0};
  for (int kk = 23; kk >= 1; --kk) {                        // sum_{k>=1} s^(2k) / (2k+1), nested
    dd kd = {(double)(2 * kk + 1), 0.0};
    dd one_over = dd_div(dd{1.0, 0.0}, kd);
    acc = dd_mul(s2, dd_add(one_over, acc));
  }
  dd lnm = dd_mul_d(dd_mul(sv, dd_add_d(acc, 1.0)), 2.0);    // 2 s (1 + s^2/3 + s^4/5 + ...)
  const double ed = (double)e;
  dd lnx = dd_two_prod(ed, RTK_LN2_A);
  lnx = dd_add(lnx, dd_two_prod(ed, RTK_LN2_B));
  lnx = dd_add_d(lnx, ed * RTK_LN2_C);
  lnx = dd_add(lnx, lnm);
  const dd L = dd_mul_d(lnx, (double)yf);
  const double n = rint(L.hi * RTK_LOG2E);
  dd r = dd_two_prod(-n, RTK_LN2_A);
  r = dd_add(r, L);
  r = dd_add(r, dd_two_prod(-n, RTK_LN2_B));
  r = dd_add_d(r, -n * RTK_LN2_C);
  dd sq = {r.hi * 0.00390625, r.lo * 0.00390625};
  dd h = {1.0, 0.0};
  for (int kk = 12; kk >= 2; --kk) {
    dd kd = {(double)kk, 0.0};
    h = dd_add_d(dd_div(dd_mul(sq, h), kd), 1.0);
  }
  dd q = dd_mul(sq, h);
  for (int i = 0; i < 8; ++i) {
    dd q2 = dd_mul(q, q);
    q = dd_add(dd_mul_d(q, 2.0), q2);
  }
  const double sc = ldexp(1.0, (int)n);
  return dd_round_f32(dd_mul_d(dd_add_d(q, 1.0), sc));
}

__device__ __forceinline__ float pow_f32_cr(float xf, float yf) {
  if (xf == 0.0f) return 0.0f;
  double m; int e;
  split_m_e(xf, &m, &e);
  const double sv = (m - 1.0) / (m + 1.0);
  const double s2 = sv * sv;
  double p = 1.0 / 25.0;
  p = __fma_rn(p, s2, 1.0 / 23.0);
  p = __fma_rn(p, s2, 1.0 / 21.0);
  p = __fma_rn(p, s2, 1.0 / 19.0);
  p = __fma_rn(p, s2, 1.0 / 17.0);
  p = __fma_rn(p, s2, 1.0 / 15.0);
  p = __fma_rn(p, s2, 1.0 / 13.0);
  p = __fma_rn(p, s2, 1.0 / 11.0);
  p = __fma_rn(p, s2, 1.0 / 9.0);
  p = __fma_rn(p, s2, 1.0 / 7.0);
  p = __fma_rn(p, s2, 1.0 / 5.0);
  p = __fma_rn(p, s2, 1.0 / 3.0);
  const double lnm = 2.0 * __fma_rn(sv * s2, p, sv);        // 2 atanh(s)
  const double ed = (double)e;
  const double lnx = __fma_rn(ed, RTK_LN2_A, __fma_rn(ed, RTK_LN2_B, lnm));
  const double L = (double)yf * lnx;
  const double n = rint(L * RTK_LOG2E);
  double r = __fma_rn(-n, RTK_LN2_A, L);
  r = __fma_rn(-n, RTK_LN2_B, r);
  double pe = 1.0 / 87178291200.0;                      // 1/14!
  pe = __fma_rn(pe, r, 1.0 / 6227020800.0);
  pe = __fma_rn(pe, r, 1.0 / 479001600.0);
  pe = __fma_rn(pe, r, 1.0 / 39916800.0);
  pe = __fma_rn(pe, r, 1.0 / 3628800.0);
  pe = __fma_rn(pe, r, 1.0 / 362880.0);
  pe = __fma_rn(pe, r, 1.0 / 40320.0);
  pe = __fma_rn(pe, r, 1.0 / 5040.0);
  pe = __fma_rn(pe, r, 1.0 / 720.0);
  pe = __fma_rn(pe, r, 1.0 / 120.0);
  pe = __fma_rn(pe, r, 1.0 / 24.0);
  pe = __fma_rn(pe, r, 1.0 / 6.0);
  pe = __fma_rn(pe, r, 0.5);
  const double q = __fma_rn(r * r, pe, r);              // expm1(r)
  const double sc = ldexp(1.0, (int)n);
  const double y = __fma_rn(sc, q, sc);                 // exp(L)
  const float lo = (float)(y * (1.0 - 0x1p-42));
  const float hi = (float)(y * (1.0 + 0x1p-42));
  if (lo == hi) return lo;
  return pow_f32_dd(xf, yf);
}

}  // namespace rtk
