// fp32 transcendental functors that must land within 2 ulp of the correctly
// rounded result.  sigmoid, tanh and gelu are composed in binary64 (the chip's
// fp64 vector rate is half its fp32 rate, and these kernels are HBM-bound), so
// the only rounding that matters is the final conversion to fp32.
#pragma once
#include "common.h"

namespace tx {

// a * b + k with the constant k read from a scalar register pair.  Left to itself the compiler turns a Horner step
// with a constant addend into the two-operand multiply-add, whose addend register is overwritten, so it first
// copies the constant into a fresh vector register pair: two moves per coefficient, which was 47 of the 105 vector
// instructions per element of the fp32 gelu.  The three-operand form reads the constant where it is.
__device__ __forceinline__ double fma_k(double a, double b, double k) {
  double r;
  asm("v_fma_f64 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "s"(k));
  return r;
}

// 1/x to ~1e-14 relative: hardware reciprocal estimate (about 24 bits) + one Newton step
// a b + 1 and a k + 1 with the 1 as the instruction's inline constant (left to itself the compiler loads it into a
// register pair and uses the two-operand form)
__device__ __forceinline__ double fma_1(double a, double b) {
  double r;
  asm("v_fma_f64 %0, %1, %2, 1.0" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ double fma_k1(double a, double k) {
  double r;
  asm("v_fma_f64 %0, %1, %2, 1.0" : "=v"(r) : "v"(a), "s"(k));
  return r;
}

__device__ __forceinline__ double rcp_d(double x) {
  double r = __builtin_amdgcn_rcp(x);
  return __builtin_fma(__builtin_fma(-x, r, 1.0), r, r);
}

// exp(y) = 2^n * (1 + p), r = y - n ln2, |r| <= ln2/2; *p_out receives p = expm1(r), *n_out receives n.
// Degree-10 Taylor polynomial (remainder below 3e-13 relative) and a two-part ln 2: for the callers that subtract
// afterwards (logaddexp near a + b = 0, pow through y log a).  y must be finite and within [-708, 708].
__device__ __forceinline__ void exp_parts_d(double y, double* p_out, int* n_out) {
  const double kLog2e = 1.4426950408889634074, kLn2Hi = 6.93147180369123816490e-01,
               kLn2Lo = 1.90821492927058770002e-10;
  double nf = __builtin_rint(y * kLog2e);
  double r = __builtin_fma(-nf, kLn2Hi, y);
  r = __builtin_fma(-nf, kLn2Lo, r);
  double p = 1.0 / 3628800.0;
  p = fma_k(p, r, 1.0 / 362880.0);
  p = fma_k(p, r, 1.0 / 40320.0);
  p = fma_k(p, r, 1.0 / 5040.0);
  p = fma_k(p, r, 1.0 / 720.0);
  p = fma_k(p, r, 1.0 / 120.0);
  p = fma_k(p, r, 1.0 / 24.0);
  p = fma_k(p, r, 1.0 / 6.0);
  p = fma_k(p, r, 0.5);
  p = fma_k(p, r, 1.0);
  *p_out = p * r;
  *n_out = (int)nf;
}
__device__ __forceinline__ double pow2_d(int n) {   // 2^n for n in the normal range
  return __longlong_as_double((long long)(n + 1023) << 52);
}
__device__ __forceinline__ double exp_d(double y) {  // y clamped by the caller
  double p;
  int n;
  exp_parts_d(y, &p, &n);
  return __builtin_fma(p, pow2_d(n), pow2_d(n));
}

// The same for results that are rounded to fp32 with nothing subtracted in between (sigmoid, tanh, gelu):
// p = r + r^2 Q(r) with Q of degree QDEG, fitted at Chebyshev nodes to the exponential's relative error (degree 4:
// below 3.7e-9; degree 5: below 6.1e-11, for tanh, whose small arguments see Q's own error; half an fp32 ulp is
// 3e-8), and one constant for ln 2 (n stays below 2400, so its rounding error, 5.5e-17 n, is far below the
// polynomial's).  y must be finite and within [-1600, 708].
template <int QDEG> __device__ __forceinline__ void exp_short_parts_d(double y, double* p_out, int* n_out) {
  const double kLog2e = 1.4426950408889634074, kLn2 = 6.93147180559945309417e-01;
  const double nf = __builtin_rint(y * kLog2e);
  const double r = __builtin_fma(-nf, kLn2, y);
  double q;
  if constexpr (QDEG == 4) {
    q = 1.37513947303978708e-03;
    q = fma_k(q, r, 8.36892165717010965e-03);
    q = fma_k(q, r, 4.16695338312040170e-02);
    q = fma_k(q, r, 1.66665184160031177e-01);
    q = fma_k(q, r, 4.99999885906078634e-01);
  } else {
    q = 1.98264486625870186e-04;
    q = fma_k(q, r, 1.39461602826869186e-03);
    q = fma_k(q, r, 8.33343047100944950e-03);
    q = fma_k(q, r, 4.16662683527592170e-02);
    q = fma_k(q, r, 1.66666661600924665e-01);
    q = fma_k(q, r, 5.00000007869999985e-01);
  }
  *p_out = __builtin_fma(r * r, q, r);
  *n_out = (int)nf;
}
__device__ __forceinline__ double exp6_d(double y) {   // a result below the normal range goes to 0 gradually
  double p;
  int n;
  exp_short_parts_d<4>(y, &p, &n);
  return __builtin_ldexp(1.0 + p, n);
}

// log(a) for finite, positive, normal a: a = 2^e m with m in [sqrt(1/2), sqrt 2), log m = 2 atanh(z),
// z = (m - 1) / (m + 1), |z| <= 0.1716: z (1 + w/3 + ... + w^7/15), w = z^2 (first dropped term below 4e-14 relative)
__device__ __forceinline__ double log_d(double a) {
  const double kLn2Hi = 6.93147180369123816490e-01, kLn2Lo = 1.90821492927058770002e-10;
  const long long bits = __double_as_longlong(a);
  int e = (int)((bits >> 52) & 0x7ff) - 1023;
  double m = __longlong_as_double((bits & 0x000fffffffffffffLL) | 0x3ff0000000000000LL);
  if (m > 1.4142135623730951) { m *= 0.5; ++e; }
  const double z = (m - 1.0) * rcp_d(m + 1.0);
  const double w = z * z;
  double p = 1.0 / 15.0;
  p = fma_k(p, w, 1.0 / 13.0);
  p = fma_k(p, w, 1.0 / 11.0);
  p = fma_k(p, w, 1.0 / 9.0);
  p = fma_k(p, w, 1.0 / 7.0);
  p = fma_k(p, w, 1.0 / 5.0);
  p = fma_k(p, w, 1.0 / 3.0);
  p = fma_k(p, w, 1.0);
  const double ef = (double)e;
  return __builtin_fma(ef, kLn2Hi, __builtin_fma(ef, kLn2Lo, 2.0 * z * p));
}

// log1p(t) for 0 <= t <= 1 (t is the exponential of a non-positive number): 2 atanh(t / (2 + t)) while that
// argument is small enough for the same series (it keeps full relative accuracy down to t = 0), log(1 + t) above
__device__ __forceinline__ double log1p_unit_d(double t) {
  if (t > 0.25) return log_d(1.0 + t);
  const double z = t * rcp_d(2.0 + t);
  const double w = z * z;
  double p = 1.0 / 15.0;
  p = fma_k(p, w, 1.0 / 13.0);
  p = fma_k(p, w, 1.0 / 11.0);
  p = fma_k(p, w, 1.0 / 9.0);
  p = fma_k(p, w, 1.0 / 7.0);
  p = fma_k(p, w, 1.0 / 5.0);
  p = fma_k(p, w, 1.0 / 3.0);
  p = fma_k(p, w, 1.0);
  return 2.0 * z * p;
}

// v^p for v >= 0 that came from an fp32 value (so it is zero, a normal binary64 number, +inf or NaN) and p != 0
__device__ __forceinline__ double pow_abs_d(double v, double p) {
  if (v != v) return v;
  const double inf = __builtin_inf();
  if (v == 0.0) return p > 0.0 ? 0.0 : inf;
  if (v == inf) return p > 0.0 ? inf : 0.0;
  const double y = p * log_d(v);
  if (y > 709.0) return inf;
  if (y < -708.0) return 0.0;                          // below 1e-307: nothing an fp32 result can see
  return exp_d(y);
}

// log1p(x) for an fp32 x, in binary64: 1 + x is exact there from |x| = 2^-29 up to 2^53 (an fp32 x has 24 bits), so
// log_d(1 + x) keeps full relative accuracy - for 1 + x in [sqrt 1/2, sqrt 2) its exponent term is zero and its
// series runs in x / (2 + x).  Below 2^-12 the first three terms of the series in x itself are exact to 2^-38.
// x < -1: NaN; x = -1: -inf; +inf stays; a NaN x fails the first comparison and comes out NaN.
__device__ __forceinline__ float log1p_f32(float xf) {
  const double x = (double)xf;
  const bool inside = xf > -1.0f && xf < __builtin_inff();
  const double l = log_d(inside ? 1.0 + x : 1.0);           // log_d wants a positive normal argument
  const double s = x * __builtin_fma(x, __builtin_fma(x, 1.0 / 3.0, -0.5), 1.0);
  float r = (float)(__builtin_fabsf(xf) < 0x1p-12f ? s : l);
  if (!(xf > -1.0f)) r = xf == -1.0f ? -__builtin_inff() : __uint_as_float(0x7fc00000u);
  return xf == __builtin_inff() ? xf : r;
}

// log(e^a + e^b) (base2: log2(2^a + 2^b)) = max + log1p(exp(-|a - b|)); fp32 operands, binary64 evaluation
__device__ __forceinline__ float logaddexp_f32(float a, float b, bool base2) {
  if (a != a || b != b) return __uint_as_float(0x7fc00000u);
  if (a == b && __builtin_fabsf(a) == __builtin_inff()) return a;
  const double kLn2 = 6.93147180559945309417e-01, kLog2e = 1.4426950408889634074;
  const double m = (double)(a > b ? a : b);
  double d = -__builtin_fabs((double)a - (double)b);
  if (base2) d *= kLn2;
  d = d < -700.0 ? -700.0 : d;                       // exp(-700) is far below half an ulp of 1
  const double l = log1p_unit_d(exp_d(d));
  return (float)(m + (base2 ? l * kLog2e : l));
}

// mish(x) = x tanh(log(1 + e^x)) = x n / (n + 2) with n = e^x (e^x + 2): one exponential, no cancellation
__device__ __forceinline__ float mish_f32(float xf) {
  if (xf > 20.0f) return xf;                          // 1 - tanh(...) = 2 / (n + 2) < 2^-25
  if (xf == -__builtin_inff()) return __uint_as_float(0x7fc00000u);   // -inf * 0
  const double x = (double)xf;
  const double w = exp6_d(x < -700.0 ? -700.0 : x);   // the short exponential: n / (n + 2) sees at most twice its 3.7e-9
  const double n = w * (w + 2.0);
  return (float)(x * n * rcp_d(n + 2.0));
}

// fp32 power.  Finite non-zero base and finite exponent: exp(b log|a|) in binary64 (the error of b log|a| stays
// below 1e-11 wherever the result is finite and the short exponential adds 3.7e-9: a sixteenth of an fp32 ulp), the
// sign from the exponent's parity for a
// negative base, NaN for a negative base with a non-integer exponent.  Zeros, infinities and NaNs: the device
// library's binary64 pow, which carries the C Annex F table.
__device__ __forceinline__ float pow_f32(float af, float bf) {
  const float aa = __builtin_fabsf(af), inf = __builtin_inff();
  if (!(aa > 0.0f && aa < inf && __builtin_fabsf(bf) < inf)) return (float)pow((double)af, (double)bf);
  if (bf == 0.0f) return 1.0f;
  bool odd = false;
  if (af < 0.0f) {
    if (bf != __builtin_truncf(bf)) return __uint_as_float(0x7fc00000u);
    odd = __builtin_fabsf(bf) < 16777216.0f && ((long long)bf & 1);      // every float from 2^24 on is an even integer
  }
  double y = (double)bf * log_d((double)aa);
  y = y > 90.0 ? 90.0 : (y < -110.0 ? -110.0 : y);                       // beyond fp32's range either way
  const float r = (float)exp6_d(y);                                      // nothing is subtracted afterwards: the short form serves
  return odd ? -r : r;
}

// 1 / (1 + exp(-x)): the exponent is clamped to where the fp32 result has long been 1 or 0.  The clamp is one
// median-of-three, which drops a NaN, so a NaN input is put back at the end.
__device__ __forceinline__ float sigmoid_f32(float xf) {
  const double y = (double)__builtin_amdgcn_fmed3f(-xf, -40.0f, 110.0f);
  const float r = (float)rcp_d(1.0 + exp6_d(y));
  return xf != xf ? xf : r;
}

// x / (1 + exp(-x)) in binary64: for large negative x the fp32 sigmoid is subnormal and would lose the product's bits
__device__ __forceinline__ float silu_f32(float xf) {
  if (xf != xf) return xf;
  if (xf == -__builtin_inff()) return __uint_as_float(0x7fc00000u);      // -inf / inf
  const double x = (double)xf;
  const double m = -x > 708.0 ? 708.0 : (-x < -708.0 ? -708.0 : -x);
  return (float)(x * rcp_d(1.0 + exp6_d(m)));
}

// tanh|x| = em / (em + 2), em = expm1(2|x|) = 2^n (1 + p) - 1 from the exponential's own reduction: with n = 0 the
// multiply-add returns p itself, so small arguments keep their relative accuracy without a branch.  The sign is copied
// at the end (keeps -0); |x| is clamped at 20, far beyond where the fp32 result is 1 (a NaN passes the clamp).
__device__ __forceinline__ float tanh_f32(float xf) {
  float ax = __builtin_fabsf(xf);
  ax = ax > 20.0f ? 20.0f : ax;
  double p;
  int n;
  exp_short_parts_d<5>(2.0 * (double)ax, &p, &n);
  const double s = pow2_d(n);
  const double em = __builtin_fma(p, s, s - 1.0);
  return __builtin_copysignf((float)(em * rcp_d(em + 2.0)), xf);
}

// gelu(x) = x Phi(x), Phi(x) = erfc(-x / sqrt 2) / 2.  With z = |x| / sqrt 2, h = Phi(-|x|) = erfc(z) / 2 is
// exp(-z^2) P(t) / (z + 3), t = (z - 3) / (z + 3) = 1 - 6 / (z + 3); P has degree 9 (relative error of h below 3.2e-9
// for z <= 10.5, where the fp32 result has already underflowed to zero; fitted at Chebyshev nodes against 40-digit
// values, the factor 1/2 folded in).  Then gelu(x) = g + max(x, 0) with g = gelu(-|x|) = -|x| h: for x >= 0 that is
// x - x h = x (1 - h), and there is one rounding to fp32 at the end.  The infinities are put in at the end (+inf,
// and the NaN that the IEEE evaluation of x Phi(x) gives at -inf); a NaN input stays NaN through -|x| h.
// All of it runs in w = z sqrt(log2 e), so that exp(-z^2) = 2^(-w^2) needs no multiplication by log2 e: with
// K = 3 sqrt(log2 e) and r = 1 / (w + K), t = 1 - 2 K r, 1 / (z + 3) = sqrt(log2 e) r (the factor sits in P's
// coefficients, beside the 1/2), and 2^(-w^2) = 2^n (1 + f S(f)) with n = round(-w^2), f = -w^2 - n in
// [-1/2, 1/2] and S of degree 5 fitted at Chebyshev nodes to the relative error of 2^f (2.2e-9).
// The leading coefficients of the two polynomials, held in vector registers: a caller that evaluates several elements
// fetches them once (gelu_lead) - the empty asm keeps the compiler from re-creating them with two moves per use.
struct GeluLead {
  double p9, q5;
};
__device__ __forceinline__ GeluLead gelu_lead() {
  GeluLead k{-1.96476019080543929e-04, 1.53707048334774087e-04};
  asm("" : "+v"(k.p9), "+v"(k.q5));
  return k;
}
// The two factors of h = erfc(z) / 2 = 2^(-w^2) (P(t) r) for w = z sqrt(log2 e) >= 0: P(t) with r = 1 / (w + K) ...
__device__ __forceinline__ double half_erfc_poly_w(double w, const GeluLead k, double* r_out) {
  const double r = rcp_d(w + 3.60336722635934947e+00);
  const double t = fma_k1(r, -7.20673445271869895e+00);
  double p = k.p9;
  p = fma_k(p, t, -2.91349187931495444e-04);
  p = fma_k(p, t, 1.85101994782671270e-03);
  p = fma_k(p, t, -7.35328772653825731e-04);
  p = fma_k(p, t, -1.61192822422337248e-02);
  p = fma_k(p, t, 7.17841652525249146e-02);
  p = fma_k(p, t, -1.86453799824604027e-01);
  p = fma_k(p, t, 3.54468249028774052e-01);
  p = fma_k(p, t, -5.30532458571298382e-01);
  p = fma_k(p, t, 6.45006881663682696e-01);
  *r_out = r;
  return p;
}
// ... and 2^(-w^2); a result below the normal range goes to 0 gradually, and a huge finite w needs no clamp: -w^2 is
// then an integer, f = 0, the conversion of n saturates and ldexp returns 0
__device__ __forceinline__ double exp2_neg_sq_w(double w, const GeluLead k) {
  const double y = -w * w;
  const double nf = __builtin_rint(y);
  const double f = y - nf;
  double q = k.q5;
  q = fma_k(q, f, 1.33998482906884158e-03);
  q = fma_k(q, f, 9.61837325129530525e-03);
  q = fma_k(q, f, 5.55032903515319184e-02);
  q = fma_k(q, f, 2.40226484622816677e-01);
  q = fma_k(q, f, 6.93147205577100745e-01);
  return __builtin_ldexp(fma_1(q, f), (int)nf);
}
__device__ __forceinline__ float gelu_erf_f32(float xf, const GeluLead k = GeluLead{-1.96476019080543929e-04, 1.53707048334774087e-04}) {
  const double x = (double)xf;
  const double w = __builtin_fabs(x) * 8.49321800288019069e-01;
  double r;
  const double p = half_erfc_poly_w(w, k, &r);
  const double e = exp2_neg_sq_w(w, k);
  // max(x, 0); a NaN x gives 0, and the product below is NaN.  (One instruction: the builtin first canonicalises x
  // with a max of its own, which a value that comes from a conversion does not need.)
  double m;
  asm("v_max_f64 %0, %1, 0" : "=v"(m) : "v"(x));
  const double a = __builtin_fabs(x) * e;                              // h = Phi(-|x|) = exp(-z^2) (p r); g = -|x| h
  // gelu(x) has the sign of x everywhere, also where it rounds to zero; copying the sign settles -0 + +0
  const float res = __builtin_copysignf((float)__builtin_fma(-a, p * r, m), xf);
  return xf == __builtin_inff() ? xf : (xf == -__builtin_inff() ? __uint_as_float(0x7fc00000u) : res);
}

// erf(x) from the same two factors with z = |x| (so w = |x| sqrt(log2 e)): 1 - 2 h, with the sign of x, from
// |x| = 1/4 on, where h <= 0.37 carries its 3.2e-9 relative error into 1 - 2 h as at most 8e-9 of the result; below
// that the Maclaurin series x (c0 + c1 x^2 + ... + c6 x^12), whose first dropped term is 5e-14 of the result there.
// |x| is clamped at 6 (erf rounds to 1 in fp32 from 3.93 on; the clamp also keeps the infinities out of -w^2 - n);
// a NaN x is returned as it is.
__device__ __forceinline__ float erf_f32(float xf, const GeluLead k = GeluLead{-1.96476019080543929e-04, 1.53707048334774087e-04}) {
  const double x = (double)xf;
  double ax = __builtin_fabs(x);
  ax = ax < 6.0 ? ax : 6.0;
  const double w = ax * 1.20112240878644982e+00;
  double r;
  const double p = half_erfc_poly_w(w, k, &r);
  const double e = exp2_neg_sq_w(w, k);
  const double tail = __builtin_fma(-2.0 * e, p * r, 1.0);
  const double u = ax * ax;
  double c = 1.20553329817896636e-04;
  c = fma_k(c, u, -8.54832702345085333e-04);
  c = fma_k(c, u, 5.22397762544218793e-03);
  c = fma_k(c, u, -2.68661706451312522e-02);
  c = fma_k(c, u, 1.12837916709551261e-01);
  c = fma_k(c, u, -3.76126389031837538e-01);
  c = fma_k(c, u, 1.12837916709551256e+00);
  const float res = __builtin_copysignf((float)(ax < 0.25 ? ax * c : tail), xf);
  return xf != xf ? xf : res;
}

// log(sigmoid(x)) = min(x, 0) - log1p(e), e = exp(-|x|) in (0, 1], composed in binary64 like the functions above.
// e comes from the short exponential (3.7e-9 relative: where log1p(e) is all of the result, for large x, it is e
// itself to first order, and elsewhere it is the smaller term).  log1p(e) = 2 atanh(z) with z = e / (2 + e) <= 1/3:
// z (1 + w/3 + w^2/5 + ... + w^8/17), w = z^2 <= 1/9; the dropped terms sum to 1.6e-9 relative at most.
// |x| is clamped at 104, where e is below half the smallest fp32 subnormal.
__device__ __forceinline__ float logsigmoid_f32(float xf) {
  if (xf != xf) return xf;
  const double x = (double)xf;
  double m = -__builtin_fabs(x);
  m = m < -104.0 ? -104.0 : m;
  const double e = exp6_d(m);
  const double z = e * rcp_d(2.0 + e);
  const double w = z * z;
  double p = 1.0 / 17.0;
  p = fma_k(p, w, 1.0 / 15.0);
  p = fma_k(p, w, 1.0 / 13.0);
  p = fma_k(p, w, 1.0 / 11.0);
  p = fma_k(p, w, 1.0 / 9.0);
  p = fma_k(p, w, 1.0 / 7.0);
  p = fma_k(p, w, 1.0 / 5.0);
  p = fma_k(p, w, 1.0 / 3.0);
  p = fma_k(p, w, 1.0);
  const double l1p = 2.0 * z * p;
  return (float)((x < 0.0 ? x : 0.0) - l1p);
}

// the same for fp16 / bf16 results in plain fp32: log1p(e) = log(u) e / (u - 1) with u = 1 + e rounded (exact
// when u == 1), hardware exp2 / log2
__device__ __forceinline__ float logsigmoid_half(float x) {
  const float e = __expf(-__builtin_fabsf(x));
  const float u = 1.0f + e;
  const float l1p = u == 1.0f ? e : __logf(u) * e * __builtin_amdgcn_rcpf(u - 1.0f);
  return __builtin_fminf(x, 0.0f) - l1p;
}

// one term of binary_cross_entropy: -(t max(ln x, -100) + (1 - t) max(ln(1 - x), -100)) in fp32.
// log(1 - x) as log1p(-x): log(u) * (-x) / (u - 1) with u = 1 - x rounded recovers the bits the rounding of u
// dropped (exact when u == 1)
__device__ __forceinline__ float log1m(float x) {
  const float u = 1.0f - x;
  return u == 1.0f ? -x : logf(u) * (-x) / (u - 1.0f);
}
__device__ __forceinline__ float bce_term(float x, float t) {
  float lx = logf(x), l1 = log1m(x);
  lx = lx < -100.0f ? -100.0f : lx;                  // written so that a NaN stays a NaN
  l1 = l1 < -100.0f ? -100.0f : l1;
  return -(t * lx + (1.0f - t) * l1);
}

// the same with the hardware log2 and reciprocal: for sums of many terms, where a term near zero (input within a
// few ulp of the target) may carry a larger relative error because it does not matter to the sum
__device__ __forceinline__ float bce_term_fast(float x, float t) {
  const float u = 1.0f - x;
  float lx = __logf(x);
  float l1 = u == 1.0f ? -x : __logf(u) * (-x) * __builtin_amdgcn_rcpf(u - 1.0f);
  lx = lx < -100.0f ? -100.0f : lx;
  l1 = l1 < -100.0f ? -100.0f : l1;
  return -(t * lx + (1.0f - t) * l1);
}

// gelu for fp16 / bf16 results (8-11 significant bits): the same erfc form in plain fp32 with a degree-5
// fit at Chebyshev nodes (relative error 5.5e-5) and the hardware exp2 / reciprocal.  Everything runs in
// w = z sqrt(log2 e), so that exp(-z^2) is the hardware's 2^(-w^2) with no further multiplication:
// t = (z - 1.5) / (z + 1.5) = 1 - 2 K r with K = 1.5 sqrt(log2 e) and r = 1 / (w + K), and the fit's coefficients
// carry the factors 1/2 and sqrt(log2 e) that turn r into 1 / (z + 1.5) and erfc into erfc / 2.
__device__ __forceinline__ float gelu_erf_half(float x) {
  const float w = __builtin_fminf(__builtin_fabsf(x) * 0.8493218002880191f, 15.614591f);      // 2^(-15.6^2) is 0 in fp32
  const float r = __builtin_amdgcn_rcpf(w + 1.8016836131796747f);
  const float t = __builtin_fmaf(-3.6033672263593495f, r, 1.0f);
  float p = -4.013620941e-03f;
  p = __builtin_fmaf(p, t, -4.943465398e-03f);
  p = __builtin_fmaf(p, t, 2.789373016e-02f);
  p = __builtin_fmaf(p, t, 4.537317152e-02f);
  p = __builtin_fmaf(p, t, -3.048984958e-01f);
  p = __builtin_fmaf(p, t, 5.793991491e-01f);
  const float half_erfc = __builtin_amdgcn_exp2f(-w * w) * p * r;
  const float phi = x < 0.0f ? half_erfc : 1.0f - half_erfc;
  return x * phi;
}

}  // namespace tx
