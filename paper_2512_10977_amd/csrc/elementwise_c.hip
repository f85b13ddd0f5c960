// Elementwise operators, third translation unit: sin cos exp2 log2 log10 rsqrt
// reciprocal silu square sign floor ceil trunc round, isnan isinf isfinite,
// bitwise_not; bitwise_and / or / xor and atan2.  One functor per family with
// the operator as a wave-uniform run-time code, so the whole batch costs a
// handful of kernel sets.
#include "ew_impl.h"

namespace tx {
namespace {

// fp32 value of a float-result operator (fp32 results within 2 ulp; half results are rounded from this)
__device__ __forceinline__ float float_op(int op, float x, bool half) {
  switch (op) {
    case TX_SIN: return sinf(x);
    case TX_COS: return cosf(x);
    case TX_EXP2: return exp2f(x);
    case TX_LOG2: return log2f(x);
    case TX_LOG10: return log10f(x);
    case TX_RSQRT: return 1.0f / sqrtf(x);
    case TX_RECIPROCAL: return 1.0f / x;
    case TX_SILU: return half ? x / (1.0f + __expf(-x)) : silu_f32(x);
    case TX_SQUARE: return x * x;
    case TX_SIGN: return (float)((0.0f < x) - (x < 0.0f));           // 0 for a NaN and for either zero
    case TX_FLOOR: return __builtin_floorf(x);
    case TX_CEIL: return __builtin_ceilf(x);
    case TX_TRUNC: return __builtin_truncf(x);
    default: return __builtin_rintf(x);                              // TX_ROUND: halves to even
  }
}

// floating tensor, out of the same dtype
template <class T> struct FloatOp {
  using Out = T; using In0 = T; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op;
  __device__ __forceinline__ T operator()(T x) const { return cvt<T>(float_op(op, cvt<float>(x), sizeof(T) == 2)); }
};
// bool / integer input (computes and returns fp32), or an out tensor of another floating dtype
struct FloatOpDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op, rd;
  __device__ __forceinline__ float operator()(float x) const { return quantize(float_op(op, x, rd != TX_F32), rd); }
};
// bool / integer tensors: square, sign, bitwise_not, and floor / ceil / trunc / round as the identity
struct IntOpDyn {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op, in_dtype, rd;
  __device__ __forceinline__ int64_t operator()(int64_t x) const {
    int64_t r = x;
    if (op == TX_SQUARE) r = (int64_t)((uint64_t)x * (uint64_t)x);
    else if (op == TX_SIGN) r = (x > 0) - (x < 0);
    else if (op == TX_BITWISE_NOT) r = in_dtype == TX_BOOL ? (int64_t)!x : ~x;
    return rd == TX_I32 ? (int64_t)(int32_t)r : r;
  }
};
// isnan / isinf / isfinite of any dtype (an integer converts to a finite float)
struct ClassifyOp {
  using Out = Dyn<int64_t>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int op;
  __device__ __forceinline__ int64_t operator()(float x) const {
    const bool nan = x != x, inf = __builtin_fabsf(x) == __builtin_inff();
    return op == TX_ISNAN ? nan : op == TX_ISINF ? inf : !(nan || inf);
  }
};

struct BitwiseDyn {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = Dyn<int64_t>; using In2 = void;
  static constexpr int NIN = 2;
  int op, common;
  __device__ __forceinline__ int64_t operator()(int64_t a, int64_t b) const {
    if (common == TX_I32) { a = (int32_t)a; b = (int32_t)b; }       // a bool operand is 0 / 1 in either width
    return op == TX_BITWISE_AND ? (a & b) : op == TX_BITWISE_OR ? (a | b) : (a ^ b);
  }
};
struct Atan2F32 {
  using Out = float; using In0 = float; using In1 = float; using In2 = void;
  static constexpr int NIN = 2;
  // the fp32 library routine reaches 3 ulp; the binary64 one rounded to fp32 stays inside 1
  __device__ __forceinline__ float operator()(float a, float b) const { return (float)atan2((double)a, (double)b); }
};
struct Atan2Dyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  int common;
  __device__ __forceinline__ float operator()(float a, float b) const {
    a = quantize(a, common);
    b = quantize(b, common);
    return common == TX_F32 ? (float)atan2((double)a, (double)b) : quantize(atan2f(a, b), common);
  }
};

}  // namespace

tx_status ew_unary_third(const Iter& it, int op, int in_dtype, int rd, hipStream_t s) {
  if (op == TX_ISNAN || op == TX_ISINF || op == TX_ISFINITE) return launch_ew(it, ClassifyOp{op}, s);
  if (!dtype_is_float(rd)) return launch_ew(it, IntOpDyn{op, in_dtype, rd}, s);
  if (in_dtype == rd && it.op[0].dtype == rd) {
    if (rd == TX_F32) return launch_ew(it, FloatOp<float>{op}, s);
    if (rd == TX_BF16) return launch_ew(it, FloatOp<bf16>{op}, s);
    return launch_ew(it, FloatOp<f16>{op}, s);
  }
  return launch_ew(it, FloatOpDyn{op, rd}, s);
}

tx_status ew_binary_third(const Iter& it, int op, int da, int db, int common, hipStream_t s) {
  if (op != TX_ATAN2) return launch_ew(it, BitwiseDyn{op, common}, s);
  if (da == TX_F32 && db == TX_F32 && it.op[0].dtype == TX_F32) return launch_ew(it, Atan2F32{}, s);
  return launch_ew(it, Atan2Dyn{common}, s);
}

}  // namespace tx
