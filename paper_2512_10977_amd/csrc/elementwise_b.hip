// Elementwise operators, second translation unit: pow, clamp, logical_not, and
// the run-time-typed forms that write a result into an out tensor of another
// dtype (`out=` casting, in-place variants).  The casting forms favour one
// kernel set per family over one per dtype: they are the rare case.
#include "ew_impl.h"

namespace tx {
namespace {

// ---------------------------------------------------------------------------
// pow
// ---------------------------------------------------------------------------

// wrapping integer power by squaring; a negative exponent is the truncated reciprocal
__device__ __forceinline__ int64_t pow_int(int64_t b, int64_t e) {
  if (e < 0) return b == 1 ? 1 : (b == -1 ? ((e & 1) ? -1 : 1) : 0);
  uint64_t r = 1, m = (uint64_t)b;
  for (uint64_t k = (uint64_t)e; k; k >>= 1) {
    if (k & 1) r *= m;
    m *= m;
  }
  return (int64_t)r;
}

struct PowF32 {
  using Out = float; using In0 = float; using In1 = float; using In2 = void;
  static constexpr int NIN = 2;
  __device__ __forceinline__ float operator()(float a, float b) const { return pow_f32(a, b); }
};
// any operand / out dtypes with a floating common dtype; a half common dtype computes in fp32
struct PowDynFloat {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  int common;
  __device__ __forceinline__ float operator()(float a, float b) const {
    a = quantize(a, common);
    b = quantize(b, common);
    return common == TX_F32 ? pow_f32(a, b) : quantize(powf(a, b), common);
  }
};
struct PowDynInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = Dyn<int64_t>; using In2 = void;
  static constexpr int NIN = 2;
  int common;
  __device__ __forceinline__ int64_t operator()(int64_t a, int64_t b) const {
    if (common == TX_I32) { a = (int32_t)a; b = (int32_t)b; }
    const int64_t r = pow_int(a, b);
    return common == TX_I32 ? (int64_t)(int32_t)r : r;
  }
};

// ---------------------------------------------------------------------------
// comparison / logical family into a non-bool out tensor
// ---------------------------------------------------------------------------
struct CompareCastFloat {
  using Out = Dyn<int64_t>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  int common, code;
  __device__ __forceinline__ int64_t operator()(float a, float b) const {
    return compare(code, quantize(a, common), quantize(b, common));
  }
};
struct CompareCastInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = Dyn<int64_t>; using In2 = void;
  static constexpr int NIN = 2;
  int common, code;
  __device__ __forceinline__ int64_t operator()(int64_t a, int64_t b) const {
    if (common == TX_I32) { a = (int32_t)a; b = (int32_t)b; }
    return compare(code, a, b);
  }
};

// ---------------------------------------------------------------------------
// unary ops with run-time dtypes
// ---------------------------------------------------------------------------
// every float-result unary op, the op chosen by a wave-uniform switch.  `half`: the result dtype is fp16 / bf16
// (cheap fp32 forms, result rounded to that dtype before the cast to out's).
struct UnaryCastFloat {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op, rd;
  __device__ __forceinline__ float operator()(float x) const {
    const bool half = rd != TX_F32;
    float r;
    switch (op) {
      case TX_NEG: r = -x; break;
      case TX_ABS: r = __builtin_fabsf(x); break;
      case TX_EXP: r = OpExp::run(x); break;
      case TX_LOG: r = OpLog::run(x); break;
      case TX_SQRT: r = OpSqrt::run(x); break;
      case TX_SIGMOID: r = half ? OpSigmoid::run_half(x) : OpSigmoid::run(x); break;
      case TX_TANH: r = half ? OpTanh::run_half(x) : OpTanh::run(x); break;
      case TX_GELU_ERF: r = half ? OpGelu::run_half(x) : OpGelu::run(x); break;
      case TX_LOG1P: r = OpLog1p::run(x); break;
      case TX_EXPM1: r = OpExpm1::run(x); break;
      default: r = half ? OpLogSigmoid::run_half(x) : OpLogSigmoid::run(x); break;
    }
    return quantize(r, rd);
  }
};
// neg / abs of an integer tensor into another dtype
struct IntSignCast {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int neg, rd;
  __device__ __forceinline__ int64_t operator()(int64_t x) const {
    uint64_t u = (uint64_t)x;
    if (neg || x < 0) u = 0 - u;
    return rd == TX_I32 ? (int64_t)(int32_t)u : (int64_t)u;
  }
};
struct LogicalNotFloat {
  using Out = Dyn<int64_t>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ int64_t operator()(float x) const { return x == 0.0f; }
};
struct LogicalNotInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ int64_t operator()(int64_t x) const { return x == 0; }
};

// ---------------------------------------------------------------------------
// clamp
// ---------------------------------------------------------------------------
// min(max(x, lo), hi); an absent bound is passed as -inf / +inf (floats) or the type's extreme (integers), which
// never binds.  A NaN x fails both comparisons and stays.
template <class T> struct ClampFloat {
  using Out = T; using In0 = T; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  float lo, hi;
  int all_nan;              // a bound is NaN
  __device__ __forceinline__ T operator()(T xv) const {
    float x = cvt<float>(xv);
    x = x < lo ? lo : x;
    x = x > hi ? hi : x;
    return cvt<T>(all_nan ? __uint_as_float(0x7fc00000u) : x);
  }
};
template <class T> struct ClampInt {
  using Out = T; using In0 = T; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  T lo, hi;
  __device__ __forceinline__ T operator()(T x) const {
    x = x < lo ? lo : x;
    return x > hi ? hi : x;
  }
};
// run-time dtypes: an integer x with a floating bound (fp32 result), or an out tensor of another dtype
struct ClampDynFloat {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  float lo, hi;
  int all_nan, rd;
  __device__ __forceinline__ float operator()(float x) const {
    x = quantize(x, rd);
    x = x < lo ? lo : x;
    x = x > hi ? hi : x;
    return all_nan ? __uint_as_float(0x7fc00000u) : x;
  }
};
struct ClampDynInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int64_t lo, hi;
  __device__ __forceinline__ int64_t operator()(int64_t x) const {
    x = x < lo ? lo : x;
    return x > hi ? hi : x;
  }
};

// host: a double rounded to the fp32 / bf16 / fp16 value the kernel compares with
float host_round_to(double v, int dt) {
  float f = (float)v;
  if (dt == TX_F32 || f != f) return f;
  if (dt == TX_F16) return (float)(_Float16)f;
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return f;
}

}  // namespace

tx_status ew_pow(const Iter& it, int da, int db, int common, hipStream_t s) {
  const bool plain = da == common && db == common && it.op[0].dtype == common;
  if (dtype_is_float(common)) {
    if (plain && common == TX_F32) return launch_ew(it, PowF32{}, s);
    return launch_ew(it, PowDynFloat{common}, s);
  }
  return launch_ew(it, PowDynInt{common}, s);
}

tx_status ew_compare_cast(const Iter& it, int code, int common, hipStream_t s) {
  if (dtype_is_float(common)) return launch_ew(it, CompareCastFloat{common, code}, s);
  return launch_ew(it, CompareCastInt{common, code}, s);
}

tx_status ew_unary_cast(const Iter& it, int op, int in_dtype, int rd, hipStream_t s) {
  if (op == TX_LOGICAL_NOT)
    return dtype_is_float(in_dtype) ? launch_ew(it, LogicalNotFloat{}, s) : launch_ew(it, LogicalNotInt{}, s);
  if (dtype_is_float(rd)) return launch_ew(it, UnaryCastFloat{op, rd}, s);
  return launch_ew(it, IntSignCast{op == TX_NEG, rd}, s);
}

}  // namespace tx

extern "C" {

tx_status tx_clamp(const tx_tensor* out, const tx_tensor* x, int has_lo, double lo_f, int64_t lo_i, int lo_is_int,
                   int has_hi, double hi_f, int64_t hi_i, int hi_is_int, void* stream) {
  using namespace tx;
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x"))) return rc;
  const int32_t rd = tx_infer_clamp_dtype(x->dtype, has_lo, lo_is_int, has_hi, hi_is_int);
  if (rd < 0) return rd;
  if (!can_cast(rd, out->dtype))
    return fail(TX_ERR_DTYPE, "a %s result cannot be written to a %s out tensor", dtype_name(rd), dtype_name(out->dtype));
  if (!same_sizes(out, x->ndim, x->sizes)) return fail(TX_ERR_SHAPE, "out does not have x's shape");
  if (rd == TX_I32 && ((has_lo && (lo_i < INT32_MIN || lo_i > INT32_MAX)) || (has_hi && (hi_i < INT32_MIN || hi_i > INT32_MAX))))
    return fail(TX_ERR_SCALAR, "clamp bound does not fit int32");
  const tx_tensor* ins[1] = {x};
  if ((rc = check_out_overlap(out, ins, 1))) return rc;
  set_path("");
  if (numel(out) == 0) return TX_OK;
  const tx_tensor* ops[2] = {out, x};
  Iter it;
  iter_build(&it, x->ndim, x->sizes, ops, 2);
  hipStream_t s = as_stream(stream);
  const bool plain = x->dtype == rd && out->dtype == rd;
  if (dtype_is_float(rd)) {
    const float inf = __builtin_inff();
    const float lo = has_lo ? host_round_to(lo_is_int ? (double)lo_i : lo_f, rd) : -inf;
    const float hi = has_hi ? host_round_to(hi_is_int ? (double)hi_i : hi_f, rd) : inf;
    const int all_nan = lo != lo || hi != hi;
    if (plain) {
      if (rd == TX_F32) return launch_ew(it, ClampFloat<float>{lo, hi, all_nan}, s);
      if (rd == TX_BF16) return launch_ew(it, ClampFloat<bf16>{lo, hi, all_nan}, s);
      return launch_ew(it, ClampFloat<f16>{lo, hi, all_nan}, s);
    }
    return launch_ew(it, ClampDynFloat{lo, hi, all_nan, rd}, s);
  }
  const int64_t lo = has_lo ? lo_i : INT64_MIN, hi = has_hi ? hi_i : INT64_MAX;
  if (plain && rd == TX_I64) return launch_ew(it, ClampInt<int64_t>{lo, hi}, s);
  if (plain && rd == TX_I32)
    return launch_ew(it, ClampInt<int32_t>{has_lo ? (int32_t)lo_i : INT32_MIN, has_hi ? (int32_t)hi_i : INT32_MAX}, s);
  return launch_ew(it, ClampDynInt{lo, hi}, s);
}

}  // extern "C"
