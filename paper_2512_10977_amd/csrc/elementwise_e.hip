// Elementwise operators, fifth translation unit: unary operators with scalar
// parameters (leaky_relu elu celu selu softplus threshold hardshrink softshrink
// logit nan_to_num) and the ternary addcmul / addcdiv / lerp.  The parameters
// are binary64 values; an fp32 result is the binary64 evaluation rounded once,
// a half result is rounded from an fp32 evaluation.
#include "ew_impl.h"

namespace tx {
namespace {

constexpr double kSeluScale = 1.0507009873554804934193349852946, kSeluAlpha = 1.6732632423543772848170429916717;

// expm1(x) for a finite or infinite x (not NaN): 2^n (1 + p) - 1 with p = expm1(r) from the exponential's own
// reduction, so small arguments keep their relative accuracy
__device__ __forceinline__ double expm1_d(double x) {
  if (x < -50.0) return -1.0;                          // below half an ulp of -1
  double p;
  int n;
  exp_parts_d(x > 700.0 ? 700.0 : x, &p, &n);          // beyond 700 the fp32 result is infinite either way
  const double s = pow2_d(n);
  return n == 0 ? p : __builtin_fma(p, s, s - 1.0);
}
// log(1 + e^y) for any y (not NaN) = max(y, 0) + log1p(e), e = exp(-|y|) in (0, 1] from the short exponential
// (3.7e-9 relative; log1p(e) is e itself to first order where it is all of the result, and the smaller term
// elsewhere).  log1p(e) = 2 atanh(z), z = e / (2 + e) <= 1/3: z (1 + w/3 + ... + w^8/17), w = z^2 <= 1/9 (the dropped
// terms sum to 1.6e-9 relative at most) - no branch between a series and a logarithm.
__device__ __forceinline__ double softplus_d(double y) {
  double t = -__builtin_fabs(y);
  t = t < -745.0 ? -745.0 : t;                         // the binary64 exponential itself has run out there
  const double e = exp6_d(t);
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
  const double l = 2.0 * z * p;
  return y > 0.0 ? y + l : l;
}

struct Params {
  int op;
  double p0, p1, p2;
};

__device__ __forceinline__ float param_op_f32(const Params& a, float xf) {
  const double x = (double)xf;
  double y;
  switch (a.op) {
    case TX_LEAKY_RELU: y = x > 0.0 ? x : x * a.p0; break;
    case TX_ELU: y = (x > 0.0 || x != x) ? x : a.p0 * expm1_d(x); break;
    case TX_CELU: y = (x > 0.0 || x != x) ? x : a.p0 * expm1_d(x / a.p0); break;
    case TX_SELU: y = kSeluScale * ((x > 0.0 || x != x) ? x : kSeluAlpha * expm1_d(x)); break;
    case TX_SOFTPLUS: {
      const double t = x * a.p0;
      y = t > a.p1 ? x : (t != t ? t : softplus_d(t) * rcp_d(a.p0));     // the reciprocal is good to 1e-14: nothing an fp32 result sees
      break;
    }
    case TX_THRESHOLD: y = x <= a.p0 ? a.p1 : x; break;              // p1 arrives rounded to the dtype
    case TX_HARDSHRINK: y = (x >= -a.p0 && x <= a.p0) ? 0.0 : x; break;
    case TX_SOFTSHRINK: y = x > a.p0 ? x - a.p0 : (x < -a.p0 ? x + a.p0 : x * 0.0); break;
    case TX_LOGIT: {
      double z = x;
      if (a.p1 != 0.0) z = z < a.p0 ? a.p0 : (z > 1.0 - a.p0 ? 1.0 - a.p0 : z);
      if (!(z >= 0.0 && z <= 1.0)) y = __builtin_nan("");
      else if (z == 0.0) y = -__builtin_inf();
      else if (z == 1.0) y = __builtin_inf();
      else y = log_d(z / (1.0 - z));
      break;
    }
    case TX_ROUND_DECIMALS: {                                         // fp32 arithmetic by definition; p1 holds 10^|d| in fp32
      const float tp = (float)a.p1;
      if (a.p0 == 0.0) return __builtin_rintf(xf);
      return a.p0 > 0.0 ? __builtin_rintf(xf * tp) / tp : __builtin_rintf(xf / tp) * tp;
    }
    case TX_GELU_TANH: {
      if (x != x) return xf;
      const double u = 0.79788456080286535588 * (x + 0.044715 * x * x * x);
      const double t = -2.0 * u;
      if (t > 700.0) return (float)(x * 0.0);                        // x / (1 + e^700): -0.0, or NaN for -inf
      y = x * rcp_d(1.0 + exp_d(t < -700.0 ? -700.0 : t));
      break;
    }
    default: y = x != x ? a.p0 : (__builtin_fabs(x) == __builtin_inf() ? (x > 0.0 ? a.p1 : a.p2) : x); break;   // TX_NAN_TO_NUM
  }
  return (float)y;
}
// for results that are rounded to 8 - 11 bits: the hardware exponential and logarithm, with two-term series where
// their absolute error would show (expm1 near 0, log1p of a small number)
__device__ __forceinline__ float expm1_half(float x) {
  return __builtin_fabsf(x) < 1e-2f ? x + 0.5f * x * x : __expf(x) - 1.0f;
}
__device__ __forceinline__ float softplus_half(float t) {            // log(1 + e^t)
  const float e = __expf(-__builtin_fabsf(t));
  const float l = e < 1e-3f ? e - 0.5f * e * e : __logf(1.0f + e);
  return t > 0.0f ? t + l : l;
}
__device__ __forceinline__ float param_op_half(const Params& a, float x) {
  const float p0 = (float)a.p0, p1 = (float)a.p1, p2 = (float)a.p2;
  switch (a.op) {
    case TX_LEAKY_RELU: return x > 0.0f ? x : x * p0;
    case TX_ELU: return x > 0.0f ? x : p0 * expm1_half(x);
    case TX_CELU: return x > 0.0f ? x : p0 * expm1_half(x / p0);
    case TX_SELU: return (float)kSeluScale * (x > 0.0f ? x : (float)kSeluAlpha * expm1_half(x));
    case TX_SOFTPLUS: {
      const float t = x * p0;
      return t > p1 ? x : softplus_half(t) / p0;
    }
    case TX_THRESHOLD: return x <= p0 ? p1 : x;
    case TX_HARDSHRINK: return (x >= -p0 && x <= p0) ? 0.0f : x;
    case TX_SOFTSHRINK: return x > p0 ? x - p0 : (x < -p0 ? x + p0 : x * 0.0f);
    case TX_LOGIT: {
      float z = x;
      if (a.p1 != 0.0) z = z < p0 ? p0 : (z > 1.0f - p0 ? 1.0f - p0 : z);
      return logf(z / (1.0f - z));
    }
    case TX_ROUND_DECIMALS:
      if (a.p0 == 0.0) return __builtin_rintf(x);
      return a.p0 > 0.0 ? __builtin_rintf(x * p1) / p1 : __builtin_rintf(x / p1) * p1;
    case TX_GELU_TANH: {
      const float t = -1.5957691216f * (x + 0.044715f * x * x * x);            // -2u
      if (t > 80.0f) return param_op_f32(a, x);                             // e^t nears fp32's range: the binary64 form keeps the tail
      return x / (1.0f + __expf(t));
    }
    default: return x != x ? p0 : (__builtin_fabsf(x) == __builtin_inff() ? (x > 0.0f ? p1 : p2) : x);
  }
}
// softplus on a plain fp32 tensor, compiled apart from the other parametrised operators (no run-time operator code,
// the reciprocal of beta computed by the host), two vectors per lane like the other composed functions
struct SoftplusF32 {
  using Out = float; using In0 = float; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  static constexpr int VPL = 2;
  double beta, inv_beta, threshold;
  __device__ __forceinline__ float operator()(float xf) const {
    const double x = (double)xf;
    const double t = x * beta;
    return (float)(t > threshold ? x : (t != t ? t : softplus_d(t) * inv_beta));
  }
};
struct ParamOpF32 {
  using Out = float; using In0 = float; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  Params a;
  __device__ __forceinline__ float operator()(float x) const { return param_op_f32(a, x); }
};
template <class T> struct ParamOpHalf {
  using Out = T; using In0 = T; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  Params a;
  __device__ __forceinline__ T operator()(T x) const { return cvt<T>(param_op_half(a, cvt<float>(x))); }
};
// logit of a bool / integer tensor (fp32 result)
struct ParamOpDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  Params a;
  int rd;
  __device__ __forceinline__ float operator()(float x) const {
    return rd == TX_F32 ? param_op_f32(a, x) : quantize(param_op_half(a, x), rd);
  }
};
// threshold (th, val already truncated to the dtype) or the identity (nan_to_num) on bool / integer tensors
struct ParamOpInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int threshold;
  int64_t th, val;
  __device__ __forceinline__ int64_t operator()(int64_t x) const { return (threshold && x <= th) ? val : x; }
};

// ---------------------------------------------------------------------------
// addcmul / addcdiv / lerp
// ---------------------------------------------------------------------------
__device__ __forceinline__ double lerp_d(double a, double b, double w) {
  return w < 0.5 ? a + w * (b - a) : b - (b - a) * (1.0 - w);
}
__device__ __forceinline__ float lerp_f(float a, float b, float w) {
  return w < 0.5f ? a + w * (b - a) : b - (b - a) * (1.0f - w);
}
struct TernaryF32 {
  using Out = float; using In0 = float; using In1 = float; using In2 = float;
  static constexpr int NIN = 3;
  int op;
  double value;
  __device__ __forceinline__ float operator()(float a, float b, float c) const {
    if (op == TX_ADDCMUL) return (float)((double)a + value * (double)b * (double)c);
    if (op == TX_ADDCDIV) return (float)((double)a + value * (double)b / (double)c);
    return (float)lerp_d(a, b, c);
  }
};
struct TernaryDynFloat {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = Dyn<float>;
  static constexpr int NIN = 3;
  int op, common;
  double value;
  __device__ __forceinline__ float operator()(float a, float b, float c) const {
    a = quantize(a, common);
    b = quantize(b, common);
    c = quantize(c, common);
    if (common == TX_F32) return TernaryF32{op, value}(a, b, c);
    const float v = (float)value;
    return quantize(op == TX_ADDCMUL ? a + v * b * c : op == TX_ADDCDIV ? a + v * b / c : lerp_f(a, b, c), common);
  }
};
struct AddcmulDynInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = Dyn<int64_t>; using In2 = Dyn<int64_t>;
  static constexpr int NIN = 3;
  int common;
  int64_t value;
  __device__ __forceinline__ int64_t operator()(int64_t a, int64_t b, int64_t c) const {
    if (common == TX_I32) { a = (int32_t)a; b = (int32_t)b; c = (int32_t)c; }
    const int64_t r = (int64_t)((uint64_t)a + (uint64_t)value * (uint64_t)b * (uint64_t)c);
    return common == TX_I32 ? (int64_t)(int32_t)r : r;
  }
};
// lerp with a scalar weight
struct LerpScalarDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  int common;
  double w;
  __device__ __forceinline__ float operator()(float a, float b) const {
    return common == TX_F32 ? (float)lerp_d(a, b, w) : quantize(lerp_f(a, b, (float)w), common);
  }
};
struct LerpScalarF32 {
  using Out = float; using In0 = float; using In1 = float; using In2 = void;
  static constexpr int NIN = 2;
  double w;
  __device__ __forceinline__ float operator()(float a, float b) const { return (float)lerp_d(a, b, w); }
};

float host_round_half(double v, int dt) {                 // a double rounded to the value the dtype holds
  float f = (float)v;
  if (dt == TX_F32 || f != f) return f;
  if (dt == TX_F16) return (float)(_Float16)f;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return f;
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return f;
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

int32_t tx_infer_unary_param_dtype(int op, int32_t in) {
  if (!dtype_valid(in)) return fail(TX_ERR_DTYPE, "unary_param: dtype code %d", in);
  switch (op) {
    case TX_LEAKY_RELU: case TX_ELU: case TX_CELU: case TX_SELU: case TX_SOFTPLUS: case TX_HARDSHRINK: case TX_SOFTSHRINK:
    case TX_ROUND_DECIMALS: case TX_GELU_TANH:
      if (!dtype_is_float(in)) return fail(TX_ERR_DTYPE, "this activation takes floating dtypes only");
      return in;
    case TX_THRESHOLD:
      if (in == TX_BOOL) return fail(TX_ERR_DTYPE, "threshold does not take bool");
      return in;
    case TX_LOGIT: return dtype_is_float(in) ? in : TX_F32;
    case TX_NAN_TO_NUM: return in;
  }
  return fail(TX_ERR_SCALAR, "unknown parametrised unary op %d", op);
}

tx_status tx_unary_param(int op, const tx_tensor* out, const tx_tensor* a, double p0, double p1, double p2, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(a, "a"))) return rc;
  const int32_t rd = tx_infer_unary_param_dtype(op, a->dtype);
  if (rd < 0) return rd;
  if (out->dtype != rd) return fail(TX_ERR_DTYPE, "out dtype %s, expected %s", dtype_name(out->dtype), dtype_name(rd));
  if (!same_sizes(out, a->ndim, a->sizes)) return fail(TX_ERR_SHAPE, "out does not have a's shape");
  if (op == TX_CELU && p0 == 0.0) return fail(TX_ERR_SCALAR, "celu: alpha must not be zero");
  if (op == TX_SOFTSHRINK && !(p0 >= 0.0)) return fail(TX_ERR_SCALAR, "softshrink: lambda must not be negative");
  if (op == TX_ROUND_DECIMALS && (p0 != std::trunc(p0) || std::fabs(p0) > 38.0))
    return fail(TX_ERR_SCALAR, "round: decimals must be an integer of magnitude at most 38");
  const tx_tensor* ins[1] = {a};
  if ((rc = check_out_overlap(out, ins, 1))) return rc;
  set_path("");
  if (numel(out) == 0) return TX_OK;
  const tx_tensor* ops[2] = {out, a};
  Iter it;
  iter_build(&it, a->ndim, a->sizes, ops, 2);
  hipStream_t s = as_stream(stream);
  if (!dtype_is_float(rd)) {
    const bool th = op == TX_THRESHOLD;
    return launch_ew(it, ParamOpInt{th, rd == TX_I32 ? (int64_t)(int32_t)p0 : (int64_t)p0, rd == TX_I32 ? (int64_t)(int32_t)p1 : (int64_t)p1}, s);
  }
  Params pa{op, p0, p1, p2};
  if (op == TX_THRESHOLD) pa.p1 = (double)host_round_half(p1, rd);
  if (op == TX_ROUND_DECIMALS) pa.p1 = (double)(float)std::pow(10.0, std::fabs(p0));
  if (op == TX_NAN_TO_NUM) { pa.p0 = (double)host_round_half(p0, rd); pa.p1 = (double)host_round_half(p1, rd); pa.p2 = (double)host_round_half(p2, rd); }
  if (a->dtype == rd) {
    if (rd == TX_F32 && op == TX_SOFTPLUS) return launch_ew(it, SoftplusF32{p0, 1.0 / p0, p1}, s);
    if (rd == TX_F32) return launch_ew(it, ParamOpF32{pa}, s);
    if (rd == TX_BF16) return launch_ew(it, ParamOpHalf<bf16>{pa}, s);
    return launch_ew(it, ParamOpHalf<f16>{pa}, s);
  }
  return launch_ew(it, ParamOpDyn{pa, rd}, s);
}

int32_t tx_infer_ternary_dtype(int op, const tx_tensor* a, const tx_tensor* b, const tx_tensor* c) {
  if (op < TX_ADDCMUL || op > TX_LERP) return fail(TX_ERR_SCALAR, "unknown ternary op %d", op);
  if (!a || !b || (op != TX_LERP && !c)) return fail(TX_ERR_NULL, "ternary: null descriptor");
  if (!dtype_valid(a->dtype) || !dtype_valid(b->dtype) || (c && !dtype_valid(c->dtype))) return fail(TX_ERR_DTYPE, "ternary: bad dtype code");
  if (op == TX_LERP) {
    if (!dtype_is_float(a->dtype) || b->dtype != a->dtype || (c && c->dtype != a->dtype))
      return fail(TX_ERR_DTYPE, "lerp takes tensors of one floating dtype");
    return a->dtype;
  }
  const tx_tensor* ops[3] = {a, b, c};
  const int rd = result_type(ops, 3);
  if (rd == TX_BOOL) return fail(TX_ERR_DTYPE, "addcmul / addcdiv do not take three bool tensors");
  if (op == TX_ADDCDIV && !dtype_is_float(rd)) return fail(TX_ERR_DTYPE, "addcdiv needs a floating operand");
  return rd;
}

tx_status tx_ternary(int op, const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, const tx_tensor* c, double value_f,
                     int64_t value_i, int value_is_int, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(a, "a")) || (rc = check_tensor(b, "b"))) return rc;
  if (c && (rc = check_tensor(c, "c"))) return rc;
  const int32_t rd = tx_infer_ternary_dtype(op, a, b, c);
  if (rd < 0) return rd;
  if (out->dtype != rd) return fail(TX_ERR_DTYPE, "out dtype %s, expected %s", dtype_name(out->dtype), dtype_name(rd));
  const tx_tensor* ins[3] = {a, b, c};
  const int nin = c ? 3 : 2;
  int nd;
  int64_t shape[TX_MAX_DIMS];
  if ((rc = broadcast_shapes(ins, nin, &nd, shape))) return rc;
  if (!same_sizes(out, nd, shape)) return fail(TX_ERR_SHAPE, "out does not have the broadcast shape");
  if ((rc = check_out_overlap(out, ins, nin))) return rc;
  set_path("");
  if (numel(out) == 0) return TX_OK;
  const tx_tensor* ops[4] = {out, a, b, c};
  Iter it;
  iter_build(&it, nd, shape, ops, nin + 1);
  hipStream_t s = as_stream(stream);
  const double value = value_is_int ? (double)value_i : value_f;
  if (!dtype_is_float(rd)) return launch_ew(it, AddcmulDynInt{rd, value_is_int ? value_i : (int64_t)value_f}, s);
  const bool plain = rd == TX_F32 && a->dtype == TX_F32 && b->dtype == TX_F32 && (!c || c->dtype == TX_F32);
  if (!c) return plain ? launch_ew(it, LerpScalarF32{value}, s) : launch_ew(it, LerpScalarDyn{rd, value}, s);
  return plain ? launch_ew(it, TernaryF32{op, value}, s) : launch_ew(it, TernaryDynFloat{op, rd, value}, s);
}

}  // extern "C"
