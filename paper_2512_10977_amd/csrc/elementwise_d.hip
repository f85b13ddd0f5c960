// Elementwise operators, fourth translation unit: tan asin acos atan sinh cosh
// asinh acosh atanh erf erfc mish (binary64 evaluation for fp32 results), relu
// frac hardswish hardsigmoid signbit; the binary fmod remainder hypot logaddexp
// logaddexp2 xlogy, copysign heaviside fmax fmin nextafter, and the integer gcd
// lcm and shifts.  As in the third unit the operator is a wave-uniform run-time
// code inside a few functor families (split by cost, so that the cheap
// operators do not inherit the register budget of the library routines).
#include "ew_impl.h"

namespace tx {
namespace {

// ---------------------------------------------------------------------------
// unary, library routines.  An fp32 result is the binary64 routine's value rounded once (the fp32 routines do
// not all stay inside 2 ulp); a half result is rounded from the fp32 routine.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float heavy_f32(int op, float xf) {
  const double x = (double)xf;
  double y;
  switch (op) {
    case TX_TAN: y = tan(x); break;
    case TX_ASIN: y = asin(x); break;
    case TX_ACOS: y = acos(x); break;
    case TX_ATAN: y = atan(x); break;
    case TX_SINH: y = sinh(x); break;
    case TX_COSH: y = cosh(x); break;
    case TX_ASINH: y = asinh(x); break;
    case TX_ACOSH: y = acosh(x); break;
    case TX_ATANH: y = atanh(x); break;
    case TX_ERF: return erf_f32(xf);
    case TX_ERFC: y = erfc(x); break;
    default: return mish_f32(xf);                                    // TX_MISH
  }
  return (float)y;
}
__device__ __forceinline__ float heavy_half(int op, float x) {
  switch (op) {
    case TX_TAN: return tanf(x);
    case TX_ASIN: return asinf(x);
    case TX_ACOS: return acosf(x);
    case TX_ATAN: return atanf(x);
    case TX_SINH: return sinhf(x);
    case TX_COSH: return coshf(x);
    case TX_ASINH: return asinhf(x);
    case TX_ACOSH: return acoshf(x);
    case TX_ATANH: return atanhf(x);
    case TX_ERF: return erff(x);
    case TX_ERFC: return erfcf(x);
    default: return x * tanhf(log1pf(expf(x)));
  }
}
// erf and mish on a plain fp32 tensor: their own binary64 compositions, compiled apart from the library routines so
// that they do not inherit those routines' register budget, two vectors per lane like the other composed functions
template <int OP> struct OwnF32 {
  using Out = float; using In0 = float; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  static constexpr int VPL = 2;
  __device__ __forceinline__ float operator()(float x) const { return OP == TX_ERF ? erf_f32(x) : mish_f32(x); }
};
template <class T> struct HeavyOp {
  using Out = T; using In0 = T; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op;
  __device__ __forceinline__ T operator()(T x) const {
    if constexpr (sizeof(T) == 2) return cvt<T>(heavy_half(op, cvt<float>(x)));
    else return heavy_f32(op, x);
  }
};
// bool / integer input (fp32 result), or an out tensor of another floating dtype
struct HeavyOpDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op, rd;
  __device__ __forceinline__ float operator()(float x) const {
    return rd == TX_F32 ? heavy_f32(op, x) : quantize(heavy_half(op, x), rd);
  }
};

// ---------------------------------------------------------------------------
// unary, arithmetic: relu frac hardsigmoid hardswish
// ---------------------------------------------------------------------------
__device__ __forceinline__ float cheap_op(int op, float x, bool half) {
  if (op == TX_RELU) return x < 0.0f ? 0.0f : x;                    // a NaN and -0.0 stay
  if (op == TX_FRAC) return x - __builtin_truncf(x);                // exact
  if (half) {
    float t = x + 3.0f;
    t = t < 0.0f ? 0.0f : t;                                        // a NaN fails both comparisons and stays
    t = t > 6.0f ? 6.0f : t;
    return op == TX_HARDSWISH ? x * t * (1.0f / 6.0f) : t * (1.0f / 6.0f);
  }
  // fp32 result: x + 3 and x * t are exact in binary64, so the value is rounded once
  double t = (double)x + 3.0;
  t = t < 0.0 ? 0.0 : t;
  t = t > 6.0 ? 6.0 : t;
  return (float)((op == TX_HARDSWISH ? (double)x * t : t) * (1.0 / 6.0));
}
template <class T> struct CheapOp {
  using Out = T; using In0 = T; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op;
  __device__ __forceinline__ T operator()(T x) const { return cvt<T>(cheap_op(op, cvt<float>(x), sizeof(T) == 2)); }
};
struct CheapOpDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op, rd;
  __device__ __forceinline__ float operator()(float x) const { return quantize(cheap_op(op, x, rd != TX_F32), rd); }
};
struct ReluInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ int64_t operator()(int64_t x) const { return x < 0 ? 0 : x; }
};
struct SignbitFloat {
  using Out = Dyn<int64_t>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ int64_t operator()(float x) const { return __float_as_uint(x) >> 31; }   // the widening keeps the bit
};
struct SignbitInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ int64_t operator()(int64_t x) const { return x < 0; }
};

// ---------------------------------------------------------------------------
// binary, floating common dtype
// ---------------------------------------------------------------------------
// fmod remainder floor_divide trunc_divide hypot logaddexp logaddexp2 xlogy.  fmodf is exact and its result needs no more bits than the
// operands have, so remainder's one addition is the only rounding; the others go through binary64 for fp32.
__device__ __forceinline__ float bin_heavy(int op, float a, float b, bool half) {
  switch (op) {
    case TX_FMOD: return fmodf(a, b);
    case TX_REMAINDER: {
      float r = fmodf(a, b);
      if (r != 0.0f && ((r < 0.0f) != (b < 0.0f))) r += b;
      return r;
    }
    case TX_TRUNC_DIVIDE: return __builtin_truncf(a / b);         // (half formats: the caller rounds the quotient first)
    case TX_FLOOR_DIVIDE: {
      // (a - fmod(a, b)) / b is an integer up to rounding: a quotient just below an integer is not rounded up to it
      if (b == 0.0f) return a / b;
      const float mod = fmodf(a, b);
      float div = (a - mod) / b;
      if (mod != 0.0f && ((b < 0.0f) != (mod < 0.0f))) div -= 1.0f;
      if (div == 0.0f) return __builtin_copysignf(0.0f, a / b);
      float fl = __builtin_floorf(div);
      if (div - fl > 0.5f) fl += 1.0f;
      return fl;
    }
    case TX_HYPOT: {
      if (__builtin_fabsf(a) == __builtin_inff() || __builtin_fabsf(b) == __builtin_inff()) return __builtin_inff();
      const double x = (double)a, y = (double)b;                   // the squares of fp32 values cannot overflow binary64
      return (float)sqrt(x * x + y * y);
    }
    case TX_XLOGY:
      if (b != b) return b;
      if (a == 0.0f) return 0.0f;
      return half ? a * logf(b) : (float)((double)a * log((double)b));
    default: {                                                       // TX_LOGADDEXP, TX_LOGADDEXP2
      if (!half) return logaddexp_f32(a, b, op == TX_LOGADDEXP2);
      if (a != a || b != b) return __uint_as_float(0x7fc00000u);
      if (a == b && __builtin_fabsf(a) == __builtin_inff()) return a;
      const float m = a > b ? a : b;
      const float d = -__builtin_fabsf(a - b);
      return op == TX_LOGADDEXP ? m + log1pf(expf(d)) : m + log1pf(exp2f(d)) * 1.44269504088896340736f;
    }
  }
}
// the neighbour of a toward b in the format `fmt`: one step on the sign-magnitude encoding
__device__ __forceinline__ float next_toward(float a, float b, int fmt) {
  if (a != a || b != b) return __uint_as_float(0x7fc00000u);
  if (a == b) return b;
  const bool away = (a < b) == (a > 0.0f);                           // the step grows the magnitude
  if (fmt == TX_F32) {
    if (a == 0.0f) return __uint_as_float((b < 0.0f ? 0x80000000u : 0u) | 1u);
    const uint32_t u = __float_as_uint(a);
    return __uint_as_float(away ? u + 1 : u - 1);
  }
  if (fmt == TX_BF16) {
    if (a == 0.0f) return __uint_as_float(((b < 0.0f ? 0x8000u : 0u) | 1u) << 16);
    const uint32_t h = __float_as_uint(a) >> 16;
    return __uint_as_float((away ? h + 1 : h - 1) << 16);
  }
  uint16_t h;
  if (a == 0.0f) h = (uint16_t)((b < 0.0f ? 0x8000u : 0u) | 1u);
  else {
    h = __builtin_bit_cast(uint16_t, (f16)a);
    h = (uint16_t)(away ? h + 1 : h - 1);
  }
  return (float)__builtin_bit_cast(f16, h);
}
// copysign heaviside fmax fmin nextafter
__device__ __forceinline__ float bin_cheap(int op, float a, float b, int fmt) {
  switch (op) {
    case TX_COPYSIGN: return __uint_as_float((__float_as_uint(a) & 0x7fffffffu) | (__float_as_uint(b) & 0x80000000u));
    case TX_HEAVISIDE: return a == 0.0f ? b : (a > 0.0f ? 1.0f : 0.0f);            // 0 for a NaN
    case TX_FMAX: return a != a ? b : (b != b ? a : (b > a ? b : a));
    case TX_FMIN: return a != a ? b : (b != b ? a : (b < a ? b : a));
    default: return next_toward(a, b, fmt);
  }
}
struct BinHeavyF32 {
  using Out = float; using In0 = float; using In1 = float; using In2 = void;
  static constexpr int NIN = 2;
  int op;
  __device__ __forceinline__ float operator()(float a, float b) const { return bin_heavy(op, a, b, false); }
};
struct BinCheapF32 {
  using Out = float; using In0 = float; using In1 = float; using In2 = void;
  static constexpr int NIN = 2;
  int op;
  __device__ __forceinline__ float operator()(float a, float b) const { return bin_cheap(op, a, b, TX_F32); }
};
// any operand / out dtypes with the floating common dtype `common`
struct BinHeavyDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  int op, common;
  __device__ __forceinline__ float operator()(float a, float b) const {
    a = quantize(a, common);
    b = quantize(b, common);
    if (op == TX_TRUNC_DIVIDE) return __builtin_truncf(quantize(a / b, common));   // truncates the quotient the format holds
    return quantize(bin_heavy(op, a, b, common != TX_F32), common);
  }
};
struct BinCheapDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  int op, common;
  __device__ __forceinline__ float operator()(float a, float b) const {
    return bin_cheap(op, quantize(a, common), quantize(b, common), common);    // every result is a value of the format
  }
};

// ---------------------------------------------------------------------------
// binary, integer / bool common dtype: fmod remainder floor_divide trunc_divide heaviside fmax fmin gcd lcm shifts
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint64_t gcd_mag(uint64_t x, uint64_t y) {
  while (y) {
    const uint64_t t = x % y;
    x = y;
    y = t;
  }
  return x;
}
struct BinIntOps {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = Dyn<int64_t>; using In2 = void;
  static constexpr int NIN = 2;
  int op, common;
  __device__ __forceinline__ int64_t operator()(int64_t a, int64_t b) const {
    const bool w32 = common == TX_I32;
    if (w32) { a = (int32_t)a; b = (int32_t)b; }
    const int width = w32 ? 32 : 64;
    int64_t r;
    switch (op) {
      case TX_FMOD: case TX_REMAINDER: {
        // a zero divisor is outside the contract: the division below is skipped for it (and for -1, where every
        // value divides and INT_MIN / -1 has no quotient) and the result is 0
        if (b == 0 || b == -1) r = 0;
        else r = w32 ? (int64_t)((int32_t)a % (int32_t)b) : a % b;
        if (op == TX_REMAINDER && r != 0 && ((r < 0) != (b < 0))) r += b;
        break;
      }
      case TX_FLOOR_DIVIDE: case TX_TRUNC_DIVIDE: {
        // a zero divisor is outside the contract (result 0); by -1 the quotient is the wrapping negation
        if (b == 0) r = 0;
        else if (b == -1) r = (int64_t)(0 - (uint64_t)a);
        else {
          r = w32 ? (int64_t)((int32_t)a / (int32_t)b) : a / b;
          if (op == TX_FLOOR_DIVIDE && r * b != a && ((a < 0) != (b < 0))) --r;
        }
        break;
      }
      case TX_HEAVISIDE: r = a == 0 ? b : (a > 0 ? 1 : 0); break;
      case TX_FMAX: r = b > a ? b : a; break;
      case TX_FMIN: r = b < a ? b : a; break;
      case TX_GCD: case TX_LCM: {
        const uint64_t ua = a < 0 ? 0 - (uint64_t)a : (uint64_t)a, ub = b < 0 ? 0 - (uint64_t)b : (uint64_t)b;
        const uint64_t g = gcd_mag(ua, ub);
        r = op == TX_GCD ? (int64_t)g : (g == 0 ? 0 : (int64_t)(ua / g * ub));
        break;
      }
      case TX_SHIFT_LEFT: r = (b < 0 || b >= width) ? 0 : (int64_t)((uint64_t)a << b); break;
      default: r = (b < 0 || b >= width) ? (a < 0 ? -1 : 0) : (a >> b); break;              // TX_SHIFT_RIGHT, arithmetic
    }
    return w32 ? (int64_t)(int32_t)r : r;
  }
};

}  // namespace

tx_status ew_unary_fourth(const Iter& it, int op, int in_dtype, int rd, hipStream_t s) {
  if (op == TX_SIGNBIT) return dtype_is_float(in_dtype) ? launch_ew(it, SignbitFloat{}, s) : launch_ew(it, SignbitInt{}, s);
  if (!dtype_is_float(rd)) return launch_ew(it, ReluInt{}, s);                     // relu of an integer tensor
  const bool plain = in_dtype == rd && it.op[0].dtype == rd;
  if (op == TX_RELU || op == TX_FRAC || op == TX_HARDSWISH || op == TX_HARDSIGMOID) {
    if (!plain) return launch_ew(it, CheapOpDyn{op, rd}, s);
    if (rd == TX_F32) return launch_ew(it, CheapOp<float>{op}, s);
    if (rd == TX_BF16) return launch_ew(it, CheapOp<bf16>{op}, s);
    return launch_ew(it, CheapOp<f16>{op}, s);
  }
  if (!plain) return launch_ew(it, HeavyOpDyn{op, rd}, s);
  if (rd == TX_F32 && op == TX_ERF) return launch_ew(it, OwnF32<TX_ERF>{}, s);
  if (rd == TX_F32 && op == TX_MISH) return launch_ew(it, OwnF32<TX_MISH>{}, s);
  if (rd == TX_F32) return launch_ew(it, HeavyOp<float>{op}, s);
  if (rd == TX_BF16) return launch_ew(it, HeavyOp<bf16>{op}, s);
  return launch_ew(it, HeavyOp<f16>{op}, s);
}

tx_status ew_binary_fourth(const Iter& it, int op, int da, int db, int common, hipStream_t s) {
  if (!dtype_is_float(common)) return launch_ew(it, BinIntOps{op, common}, s);
  const bool plain = da == TX_F32 && db == TX_F32 && it.op[0].dtype == TX_F32;
  const bool cheap = op == TX_COPYSIGN || op == TX_HEAVISIDE || op == TX_FMAX || op == TX_FMIN || op == TX_NEXTAFTER;
  if (cheap) return plain ? launch_ew(it, BinCheapF32{op}, s) : launch_ew(it, BinCheapDyn{op, common}, s);
  return plain ? launch_ew(it, BinHeavyF32{op}, s) : launch_ew(it, BinHeavyDyn{op, common}, s);
}

}  // namespace tx
