// Elementwise operators, first translation unit: unary math, add / sub / mul /
// div / maximum / minimum, the comparison and logical families, where and
// masked_fill, and the C entry points that dispatch to them.
#include "ew_impl.h"

namespace tx {
namespace {

// float math op on a statically typed float tensor (computes in fp32)
template <class Op, class T> struct MathStatic {
  using Out = T; using In0 = T; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  // two vectors per lane for the operators composed in binary64 (their arithmetic then overlaps the second vector's
  // load: gelu 108 -> 101 us, tanh 92 -> 83 us on [8192,8192] fp32), one for the cheap ones (exp: 79 against 82 us)
  static constexpr int VPL = vec_per_lane<Op>(0);
  __device__ __forceinline__ T operator()(T x) const {
    if constexpr (sizeof(T) == 2) return cvt<T>(Op::run_half(cvt<float>(x)));
    else return cvt<T>(Op::run(cvt<float>(x)));
  }
  // the fp32 operators that define run_n evaluate a whole vector at once
  template <int E, class O = Op, class = decltype(&O::template run_n<E>), class U = T, class = std::enable_if_t<sizeof(U) == 4>>
  __device__ __forceinline__ void apply_n(const T (&x)[E], T (&y)[E]) const {
    Op::template run_n<E>(x, y);
  }
};
// float math op on a bool / integer tensor: convert to fp32, fp32 result
template <class Op> struct MathDyn {
  using Out = float; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ float operator()(float x) const { return Op::run(x); }
};
// sign-bit operations on the stored encoding of a float type
template <class B, bool NEG> struct SignBits {
  using Out = B; using In0 = B; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ B operator()(B x) const {
    constexpr B sb = (B)1 << (8 * sizeof(B) - 1);
    return NEG ? (B)(x ^ sb) : (B)(x & (B)~sb);
  }
};
template <class T, bool NEG> struct IntSign {
  using Out = T; using In0 = T; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ T operator()(T x) const {
    using UT = typename std::make_unsigned<T>::type;
    UT u = (UT)x;
    if (NEG || x < 0) u = (UT)0 - u;
    return (T)u;
  }
};

// same-dtype float binary op (fp32 arithmetic, one rounding to T)
template <int OP, class T> struct BinFloat {
  using Out = T; using In0 = T; using In1 = T; using In2 = void;
  static constexpr int NIN = 2;
  float alpha;
  int flag;                 // kAdd: alpha == 1 (plain add); kMax: 1 = minimum
  __device__ __forceinline__ T operator()(T xa, T xb) const {
    float a = cvt<float>(xa), b = cvt<float>(xb), r;
    if constexpr (OP == kAdd) r = flag ? a + b : __fmaf_rn(alpha, b, a);
    else if constexpr (OP == kMul) r = a * b;
    else if constexpr (OP == kDiv) r = a / b;
    else r = flag ? fmin_nan(a, b) : fmax_nan(a, b);
    return cvt<T>(r);
  }
};
// add / mul of one fp32 operand and one half operand into an fp32 result (the promoted dtype): static operand types,
// so the loads carry no run-time dtype switch (the run-time-typed functor reaches 0.71 of peak on this pair)
template <int OP, class TA, class TB> struct BinMixedF32 {
  using Out = float; using In0 = TA; using In1 = TB; using In2 = void;
  static constexpr int NIN = 2;
  float alpha;
  int flag;                 // kAdd: alpha == 1 (plain add)
  __device__ __forceinline__ float operator()(TA xa, TB xb) const {
    const float a = cvt<float>(xa), b = cvt<float>(xb);
    if constexpr (OP == kAdd) return flag ? a + b : __fmaf_rn(alpha, b, a);
    else return a * b;
  }
};
template <class T> struct EqStatic {
  using Out = uint8_t; using In0 = T; using In1 = T; using In2 = void;
  static constexpr int NIN = 2;
  int code;                 // TX_EQ ... TX_GE
  __device__ __forceinline__ uint8_t operator()(T a, T b) const {
    if constexpr (std::is_integral<T>::value) return compare(code, a, b);
    else return compare(code, cvt<float>(a), cvt<float>(b));
  }
};
template <int OP, class T> struct BinInt {
  using Out = T; using In0 = T; using In1 = T; using In2 = void;
  static constexpr int NIN = 2;
  int64_t alpha;            // kMax: 1 = minimum
  __device__ __forceinline__ T operator()(T a, T b) const {
    using UT = typename std::make_unsigned<T>::type;
    if constexpr (OP == kAdd) return (T)((UT)a + (UT)alpha * (UT)b);
    else if constexpr (OP == kMul) return (T)((UT)a * (UT)b);
    else return alpha ? (b < a ? b : a) : (b > a ? b : a);
  }
};
template <int OP> struct BinBool {
  using Out = uint8_t; using In0 = uint8_t; using In1 = uint8_t; using In2 = void;
  static constexpr int NIN = 2;
  int flag;                 // kAdd: alpha != 0; kMax: 1 = minimum; kEq: comparison code
  __device__ __forceinline__ uint8_t operator()(uint8_t a, uint8_t b) const {
    a = a != 0; b = b != 0;
    if constexpr (OP == kAdd) return a | (b & (uint8_t)flag);
    else if constexpr (OP == kMul) return a & b;
    else if constexpr (OP == kMax) return flag ? (a & b) : (a | b);
    else return compare(flag, a, b);
  }
};
// float-result binary op with run-time operand / out dtypes (mixed operands, or an out tensor of another float
// dtype): operands converted to the common dtype first
template <int OP> struct BinDynFloat {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  float alpha;
  int flag, common;         // flag as in BinFloat
  __device__ __forceinline__ float operator()(float a, float b) const {
    a = quantize(a, common);
    b = quantize(b, common);
    float r;
    if constexpr (OP == kAdd) r = flag ? a + b : __fmaf_rn(alpha, b, a);
    else if constexpr (OP == kMul) r = a * b;
    else if constexpr (OP == kDiv) r = a / b;
    else r = flag ? fmin_nan(a, b) : fmax_nan(a, b);
    return quantize(r, common);          // the result exists in the common dtype before any cast to out's dtype
  }
};
struct EqDynFloat {
  using Out = uint8_t; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  int common, code;
  __device__ __forceinline__ uint8_t operator()(float a, float b) const {
    return compare(code, quantize(a, common), quantize(b, common));
  }
};
template <int OP> struct BinDynInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = Dyn<int64_t>; using In2 = void;
  static constexpr int NIN = 2;
  int64_t alpha;            // kMax: 1 = minimum
  int common;
  __device__ __forceinline__ int64_t operator()(int64_t a, int64_t b) const {
    if (common == TX_I32) { a = (int32_t)a; b = (int32_t)b; }
    int64_t r;
    if constexpr (OP == kAdd) r = (int64_t)((uint64_t)a + (uint64_t)alpha * (uint64_t)b);
    else if constexpr (OP == kMul) r = (int64_t)((uint64_t)a * (uint64_t)b);
    else r = alpha ? (b < a ? b : a) : (b > a ? b : a);
    // the result exists in the common dtype before any cast to out's dtype (bool: alpha is 0 or 1 here, so a sum
    // is 0..2 and "non-zero" is the OR)
    return common == TX_I32 ? (int64_t)(int32_t)r : common == TX_BOOL ? (int64_t)(r != 0) : r;
  }
};
struct EqDynInt {
  using Out = uint8_t; using In0 = Dyn<int64_t>; using In1 = Dyn<int64_t>; using In2 = void;
  static constexpr int NIN = 2;
  int common, code;
  __device__ __forceinline__ uint8_t operator()(int64_t a, int64_t b) const {
    if (common == TX_I32) { a = (int32_t)a; b = (int32_t)b; }
    return compare(code, a, b);
  }
};

// where / masked_fill on raw storage words (no conversion: bits are copied)
template <class B> struct SelectBits {
  using Out = B; using In0 = uint8_t; using In1 = B; using In2 = B;
  static constexpr int NIN = 3;
  __device__ __forceinline__ B operator()(uint8_t c, B x, B y) const { return c ? x : y; }
};
template <class CT> struct SelectDyn {
  using Out = Dyn<CT>; using In0 = uint8_t; using In1 = Dyn<CT>; using In2 = Dyn<CT>;
  static constexpr int NIN = 3;
  __device__ __forceinline__ CT operator()(uint8_t c, CT x, CT y) const { return c ? x : y; }
};
template <class B> struct FillBits {
  using Out = B; using In0 = B; using In1 = uint8_t; using In2 = void;
  static constexpr int NIN = 2;
  B value;
  __device__ __forceinline__ B operator()(B s, uint8_t m) const { return m ? value : s; }
};

// ---------------------------------------------------------------------------
// host-side scalar encoding (masked_fill value -> storage bits)
// ---------------------------------------------------------------------------
uint16_t host_float_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
uint16_t host_float_to_f16(float f) {
  _Float16 h = (_Float16)f;
  uint16_t b;
  memcpy(&b, &h, 2);
  return b;
}

template <class Op> tx_status dispatch_math(const Iter& it, int in_dtype, hipStream_t s) {
  switch (in_dtype) {
    case TX_F32: return launch_ew(it, MathStatic<Op, float>{}, s);
    case TX_BF16: return launch_ew(it, MathStatic<Op, bf16>{}, s);
    case TX_F16: return launch_ew(it, MathStatic<Op, f16>{}, s);
    default: return launch_ew(it, MathDyn<Op>{}, s);
  }
}

// `variant`: kMax: 1 = minimum; kEq: the comparison code (TX_EQ ... TX_GE); unused otherwise
template <int OP> tx_status dispatch_binary(const Iter& it, int da, int db, int common, double alpha_f, int64_t alpha_i,
                                            int alpha_is_int, hipStream_t s, int variant = 0, bool cast = false) {
  const double ad = alpha_is_int ? (double)alpha_i : alpha_f;
  const bool one = alpha_is_int ? alpha_i == 1 : alpha_f == 1.0;
  const int fflag = OP == kMax ? variant : (int)one;                 // BinFloat / BinDynFloat flag
  const int64_t ialpha = OP == kMax ? (int64_t)variant : alpha_i;     // BinInt / BinDynInt field
  // cast: out's dtype differs from the result dtype; the run-time-typed functors store into any dtype
  const bool same = da == common && db == common && !cast;
  if (dtype_is_float(common)) {
    if constexpr (OP == kEq) {
      if (cast) return ew_compare_cast(it, variant, common, s);
      if (same) {
        if (common == TX_F32) return launch_ew(it, EqStatic<float>{variant}, s);
        if (common == TX_BF16) return launch_ew(it, EqStatic<bf16>{variant}, s);
        return launch_ew(it, EqStatic<f16>{variant}, s);
      }
      return launch_ew(it, EqDynFloat{common, variant}, s);
    } else {
      if (same) {
        if (common == TX_F32) return launch_ew(it, BinFloat<OP, float>{(float)ad, fflag}, s);
        if (common == TX_BF16) return launch_ew(it, BinFloat<OP, bf16>{(float)ad, fflag}, s);
        return launch_ew(it, BinFloat<OP, f16>{(float)ad, fflag}, s);
      }
      if constexpr (OP == kAdd || OP == kMul) {
        if (common == TX_F32 && !cast) {
          if (da == TX_BF16 && db == TX_F32) return launch_ew(it, BinMixedF32<OP, bf16, float>{(float)ad, fflag}, s);
          if (da == TX_F32 && db == TX_BF16) return launch_ew(it, BinMixedF32<OP, float, bf16>{(float)ad, fflag}, s);
          if (da == TX_F16 && db == TX_F32) return launch_ew(it, BinMixedF32<OP, f16, float>{(float)ad, fflag}, s);
          if (da == TX_F32 && db == TX_F16) return launch_ew(it, BinMixedF32<OP, float, f16>{(float)ad, fflag}, s);
        }
      }
      return launch_ew(it, BinDynFloat<OP>{(float)ad, fflag, common}, s);
    }
  }
  if constexpr (OP != kDiv) {
    if constexpr (OP == kEq) {
      if (cast) return ew_compare_cast(it, variant, common, s);
    }
    const int bool_flag = OP == kAdd ? (int)(alpha_is_int ? alpha_i != 0 : alpha_f != 0.0) : variant;
    if (common == TX_BOOL && !cast) return launch_ew(it, BinBool<OP>{bool_flag}, s);
    if constexpr (OP == kEq) {
      if (same && common == TX_I32) return launch_ew(it, EqStatic<int32_t>{variant}, s);
      if (same && common == TX_I64) return launch_ew(it, EqStatic<int64_t>{variant}, s);
      return launch_ew(it, EqDynInt{common, variant}, s);
    } else {
      if (same && common == TX_I32) return launch_ew(it, BinInt<OP, int32_t>{ialpha}, s);
      if (same && common == TX_I64) return launch_ew(it, BinInt<OP, int64_t>{ialpha}, s);
      return launch_ew(it, BinDynInt<OP>{common == TX_BOOL ? (int64_t)bool_flag : ialpha, common}, s);
    }
  }
  return fail(TX_ERR_UNSUPPORTED, "no kernel for this binary op / dtype");
}

tx_status binary_impl(int op, const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, double alpha_f,
                      int64_t alpha_i, int alpha_is_int, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(a, "a")) || (rc = check_tensor(b, "b"))) return rc;
  int32_t rd, nd;
  int64_t shape[TX_MAX_DIMS];
  if ((rc = tx_infer_binary(op, a, b, &rd, &nd, shape))) return rc;
  if (!can_cast(rd, out->dtype))
    return fail(TX_ERR_DTYPE, "a %s result cannot be written to a %s out tensor", dtype_name(rd), dtype_name(out->dtype));
  const bool cast = out->dtype != rd;
  if (!same_sizes(out, nd, shape)) return fail(TX_ERR_SHAPE, "out does not have the broadcast shape");
  const tx_tensor* ins[2] = {a, b};
  int common = result_type(ins, 2);
  if ((op == TX_DIV || op == TX_ATAN2 || op == TX_COPYSIGN || op == TX_XLOGY) && !dtype_is_float(common)) common = TX_F32;
  if ((op == TX_ADD || op == TX_SUB) && !dtype_is_float(common) && !alpha_is_int)
    return fail(TX_ERR_SCALAR, "floating alpha with an integer / bool result");
  if ((rc = check_out_overlap(out, ins, 2))) return rc;
  set_path("");
  if (numel(out) == 0) return TX_OK;
  const tx_tensor* ops[3] = {out, a, b};
  Iter it;
  iter_build(&it, nd, shape, ops, 3);
  hipStream_t s = as_stream(stream);
  switch (op) {
    case TX_ADD: return dispatch_binary<kAdd>(it, a->dtype, b->dtype, common, alpha_f, alpha_i, alpha_is_int, s, 0, cast);
    case TX_MUL: return dispatch_binary<kMul>(it, a->dtype, b->dtype, common, 1.0, 1, 1, s, 0, cast);
    case TX_DIV: return dispatch_binary<kDiv>(it, a->dtype, b->dtype, common, 1.0, 1, 1, s, 0, cast);
    case TX_MAXIMUM: return dispatch_binary<kMax>(it, a->dtype, b->dtype, common, 1.0, 1, 1, s, 0, cast);
    case TX_MINIMUM: return dispatch_binary<kMax>(it, a->dtype, b->dtype, common, 1.0, 1, 1, s, 1, cast);
    // a - alpha * b = a + (-alpha) * b: one fma(-alpha, b, a) for floats (alpha = 1: the exactly rounded a - b),
    // wrapping arithmetic for integers
    case TX_SUB:
      return dispatch_binary<kAdd>(it, a->dtype, b->dtype, common, -alpha_f, (int64_t)(0 - (uint64_t)alpha_i), alpha_is_int,
                                   s, 0, cast);
    case TX_EQ: case TX_NE: case TX_LT: case TX_LE: case TX_GT: case TX_GE:
    case TX_LOGICAL_AND: case TX_LOGICAL_OR: case TX_LOGICAL_XOR:
      return dispatch_binary<kEq>(it, a->dtype, b->dtype, common, 1.0, 1, 1, s, op, cast);
    case TX_POW: return ew_pow(it, a->dtype, b->dtype, common, s);
    case TX_BITWISE_AND: case TX_BITWISE_OR: case TX_BITWISE_XOR: case TX_ATAN2:
      return ew_binary_third(it, op, a->dtype, b->dtype, common, s);
  }
  if (op >= TX_FMOD) return ew_binary_fourth(it, op, a->dtype, b->dtype, common, s);
  return fail(TX_ERR_DTYPE, "unknown binary op %d", op);
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

tx_status tx_unary(int op, const tx_tensor* out, const tx_tensor* a, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(a, "a"))) return rc;
  int32_t rd = tx_infer_unary_dtype(op, a->dtype);
  if (rd < 0) return rd;
  if (!can_cast(rd, out->dtype))
    return fail(TX_ERR_DTYPE, "a %s result cannot be written to a %s out tensor", dtype_name(rd), dtype_name(out->dtype));
  if (!same_sizes(out, a->ndim, a->sizes)) return fail(TX_ERR_SHAPE, "out does not have a's shape");
  const tx_tensor* ins[1] = {a};
  if ((rc = check_out_overlap(out, ins, 1))) return rc;
  set_path("");
  if (numel(out) == 0) return TX_OK;
  const tx_tensor* ops[2] = {out, a};
  Iter it;
  iter_build(&it, a->ndim, a->sizes, ops, 2);
  hipStream_t s = as_stream(stream);
  if (op >= TX_TAN) return ew_unary_fourth(it, op, a->dtype, rd, s);
  if (op >= TX_SIN) return ew_unary_third(it, op, a->dtype, rd, s);
  if (out->dtype != rd || op == TX_LOGICAL_NOT) return ew_unary_cast(it, op, a->dtype, rd, s);
  if (op == TX_NEG || op == TX_ABS) {
    const bool neg = op == TX_NEG;
    switch (a->dtype) {
      case TX_I32: return neg ? launch_ew(it, IntSign<int32_t, true>{}, s) : launch_ew(it, IntSign<int32_t, false>{}, s);
      case TX_I64: return neg ? launch_ew(it, IntSign<int64_t, true>{}, s) : launch_ew(it, IntSign<int64_t, false>{}, s);
      case TX_F32: return neg ? launch_ew(it, SignBits<uint32_t, true>{}, s) : launch_ew(it, SignBits<uint32_t, false>{}, s);
      default: return neg ? launch_ew(it, SignBits<uint16_t, true>{}, s) : launch_ew(it, SignBits<uint16_t, false>{}, s);
    }
  }
  switch (op) {
    case TX_EXP: return dispatch_math<OpExp>(it, a->dtype, s);
    case TX_LOG: return dispatch_math<OpLog>(it, a->dtype, s);
    case TX_SQRT: return dispatch_math<OpSqrt>(it, a->dtype, s);
    case TX_SIGMOID: return dispatch_math<OpSigmoid>(it, a->dtype, s);
    case TX_TANH: return dispatch_math<OpTanh>(it, a->dtype, s);
    case TX_GELU_ERF: return dispatch_math<OpGelu>(it, a->dtype, s);
    case TX_LOG1P: return dispatch_math<OpLog1p>(it, a->dtype, s);
    case TX_EXPM1: return dispatch_math<OpExpm1>(it, a->dtype, s);
    case TX_LOGSIGMOID: return dispatch_math<OpLogSigmoid>(it, a->dtype, s);
  }
  return fail(TX_ERR_DTYPE, "unknown unary op %d", op);
}

tx_status tx_add(const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, double alpha_f, int64_t alpha_i,
                 int alpha_is_int, void* stream) {
  return binary_impl(TX_ADD, out, a, b, alpha_f, alpha_i, alpha_is_int, stream);
}

tx_status tx_sub(const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, double alpha_f, int64_t alpha_i,
                 int alpha_is_int, void* stream) {
  return binary_impl(TX_SUB, out, a, b, alpha_f, alpha_i, alpha_is_int, stream);
}

tx_status tx_binary(int op, const tx_tensor* out, const tx_tensor* a, const tx_tensor* b, void* stream) {
  return binary_impl(op, out, a, b, 1.0, 1, 1, stream);
}

tx_status tx_where(const tx_tensor* out, const tx_tensor* cond, const tx_tensor* x, const tx_tensor* y, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(cond, "cond")) || (rc = check_tensor(x, "x")) ||
      (rc = check_tensor(y, "y")))
    return rc;
  if (cond->dtype != TX_BOOL) return fail(TX_ERR_DTYPE, "where: cond must be bool");
  const tx_tensor* xy[2] = {x, y};
  const int rd = result_type(xy, 2);
  if (out->dtype != rd) return fail(TX_ERR_DTYPE, "out dtype %s, expected %s", dtype_name(out->dtype), dtype_name(rd));
  const tx_tensor* ins[3] = {cond, x, y};
  int nd;
  int64_t shape[TX_MAX_DIMS];
  if ((rc = broadcast_shapes(ins, 3, &nd, shape))) return rc;
  if (!same_sizes(out, nd, shape)) return fail(TX_ERR_SHAPE, "out does not have the broadcast shape");
  if ((rc = check_out_overlap(out, ins, 3))) return rc;
  set_path("");
  if (numel(out) == 0) return TX_OK;
  const tx_tensor* ops[4] = {out, cond, x, y};
  Iter it;
  iter_build(&it, nd, shape, ops, 4);
  hipStream_t s = as_stream(stream);
  if (x->dtype == rd && y->dtype == rd) {
    switch (dtype_size(rd)) {
      case 1: return launch_ew(it, SelectBits<uint8_t>{}, s);
      case 2: return launch_ew(it, SelectBits<uint16_t>{}, s);
      case 4: return launch_ew(it, SelectBits<uint32_t>{}, s);
      default: return launch_ew(it, SelectBits<uint64_t>{}, s);
    }
  }
  if (dtype_is_float(rd)) return launch_ew(it, SelectDyn<float>{}, s);
  return launch_ew(it, SelectDyn<int64_t>{}, s);
}

tx_status tx_masked_fill(const tx_tensor* out, const tx_tensor* self, const tx_tensor* mask, double value_f,
                         int64_t value_i, int value_is_int, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(self, "self")) || (rc = check_tensor(mask, "mask")))
    return rc;
  if (mask->dtype != TX_BOOL) return fail(TX_ERR_DTYPE, "masked_fill: mask must be bool");
  if (out->dtype != self->dtype) return fail(TX_ERR_DTYPE, "masked_fill: out must have self's dtype");
  const tx_tensor* ins[2] = {self, mask};
  int nd;
  int64_t shape[TX_MAX_DIMS];
  if ((rc = broadcast_shapes(ins, 2, &nd, shape))) return rc;
  if (!same_sizes(out, nd, shape)) return fail(TX_ERR_SHAPE, "out does not have the broadcast shape");
  if ((rc = check_out_overlap(out, ins, 2))) return rc;
  set_path("");
  if (numel(out) == 0) return TX_OK;
  const tx_tensor* ops[3] = {out, self, mask};
  Iter it;
  iter_build(&it, nd, shape, ops, 3);
  hipStream_t s = as_stream(stream);
  const double vd = value_is_int ? (double)value_i : value_f;
  switch (self->dtype) {
    case TX_BOOL: return launch_ew(it, FillBits<uint8_t>{(uint8_t)(value_is_int ? value_i != 0 : value_f != 0.0)}, s);
    case TX_I32: {
      int32_t v = (int32_t)(uint32_t)(uint64_t)(value_is_int ? value_i : (int64_t)std::trunc(value_f));
      uint32_t b;
      memcpy(&b, &v, 4);
      return launch_ew(it, FillBits<uint32_t>{b}, s);
    }
    case TX_I64: {
      int64_t v = value_is_int ? value_i : (int64_t)std::trunc(value_f);
      uint64_t b;
      memcpy(&b, &v, 8);
      return launch_ew(it, FillBits<uint64_t>{b}, s);
    }
    case TX_F32: {
      float v = (float)vd;
      uint32_t b;
      memcpy(&b, &v, 4);
      return launch_ew(it, FillBits<uint32_t>{b}, s);
    }
    case TX_BF16: return launch_ew(it, FillBits<uint16_t>{host_float_to_bf16((float)vd)}, s);
    default: return launch_ew(it, FillBits<uint16_t>{host_float_to_f16((float)vd)}, s);
  }
}

}  // extern "C"
