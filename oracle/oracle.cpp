// CPU oracle for the ATen-operator hot path.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
// HIP library is checked against; the product never calls it.  Only the test
// suite, the smoke check and the benchmark's cpu_baseline leg load it.  It
// shares no source, header, table or helper with the HIP side.
//
// What it computes: the value an ATen operator returns on strided, typed,
// broadcast host tensors -- the "reference ATen CPU implementation" that the
// paper's test runner compares every generated kernel with (Section 3.2,
// "System Design / Agent": device output vs. CPU reference on identical
// inputs, dtype-dependent tolerance).  The paper names the operator set and
// the dtypes (Section 3.3; Table 1 categories Elementwise, Reduction,
// Indexing & Selection, and softmax from Deep Learning) and delegates the
// semantics to the PyTorch operator documentation, so every function below
// is the documented definition of its operator written out as one scalar
// loop nest over the logical index space: offset = sum_d idx[d]*stride[d].
// No blocking, no vectorisation, no reordering.
//
// Arithmetic policy:
//   * integer / bool / index results: exact two's-complement arithmetic.
//   * fp32 add / mul / where / neg / abs / maximum / eq: evaluated in IEEE
//     binary32 (a single rounding, the same one the device must produce).
//   * everything else with a floating result (div, transcendentals,
//     reductions, softmax, cumsum, scatter_add): evaluated in binary64 from
//     the (already converted) inputs and rounded ONCE to the output dtype.
//   * fp16 / bf16 operands are first read exactly into binary32; results for
//     a half output dtype are rounded once from the wider value.
// Independent output elements may be computed by different OpenMP threads;
// one accumulation is never split, so results do not depend on thread count.
//
// Parity pins: every function here is pinned by tests/test_oracle_*.py
// (closed forms, invariants, brute force, mpmath); none is "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

enum { ORC_BOOL = 0, ORC_I32 = 1, ORC_I64 = 2, ORC_F16 = 3, ORC_BF16 = 4, ORC_F32 = 5 };
enum { ORC_MAX_DIMS = 8 };

// Plain descriptor of a host tensor.  strides are in elements.
typedef struct {
  void* data;
  int32_t dtype;
  int32_t ndim;
  int64_t sizes[ORC_MAX_DIMS];
  int64_t strides[ORC_MAX_DIMS];
} orc_tensor;

// error codes (negative)
enum {
  ORC_OK = 0,
  ORC_ERR_NULL = -1,
  ORC_ERR_NDIM = -2,
  ORC_ERR_DTYPE = -3,
  ORC_ERR_SHAPE = -4,
  ORC_ERR_DIM = -5,
  ORC_ERR_EMPTY_REDUCTION = -7,
  ORC_ERR_SCALAR = -8,
  ORC_ERR_INDEX = -10,
};

// op codes
enum { ORC_NEG = 0, ORC_ABS, ORC_EXP, ORC_LOG, ORC_SQRT, ORC_SIGMOID, ORC_TANH, ORC_GELU, ORC_LOG1P, ORC_EXPM1,
       ORC_LOGSIGMOID, ORC_LOGICAL_NOT, ORC_SIN, ORC_COS, ORC_EXP2, ORC_LOG2, ORC_LOG10, ORC_RSQRT, ORC_RECIPROCAL,
       ORC_SILU, ORC_SQUARE, ORC_SIGN, ORC_FLOOR, ORC_CEIL, ORC_TRUNC, ORC_ROUND, ORC_ISNAN, ORC_ISINF, ORC_ISFINITE,
       ORC_BITWISE_NOT, ORC_TAN, ORC_ASIN, ORC_ACOS, ORC_ATAN, ORC_SINH, ORC_COSH, ORC_ASINH, ORC_ACOSH, ORC_ATANH, ORC_ERF,
       ORC_ERFC, ORC_RELU, ORC_FRAC, ORC_SIGNBIT, ORC_HARDSWISH, ORC_HARDSIGMOID, ORC_MISH };
enum { ORC_ADD = 0, ORC_MUL, ORC_DIV, ORC_MAXIMUM, ORC_EQ, ORC_SUB, ORC_MINIMUM, ORC_NE, ORC_LT, ORC_LE, ORC_GT, ORC_GE,
       ORC_LOGICAL_AND, ORC_LOGICAL_OR, ORC_LOGICAL_XOR, ORC_POW, ORC_BITWISE_AND, ORC_BITWISE_OR, ORC_BITWISE_XOR,
       ORC_ATAN2, ORC_FMOD, ORC_REMAINDER, ORC_HYPOT, ORC_COPYSIGN, ORC_LOGADDEXP, ORC_LOGADDEXP2, ORC_XLOGY, ORC_HEAVISIDE,
       ORC_FMAX, ORC_FMIN, ORC_NEXTAFTER, ORC_GCD, ORC_LCM, ORC_SHIFT_LEFT, ORC_SHIFT_RIGHT, ORC_FLOOR_DIVIDE, ORC_TRUNC_DIVIDE };
enum { ORC_LEAKY_RELU = 0, ORC_ELU, ORC_CELU, ORC_SELU, ORC_SOFTPLUS, ORC_THRESHOLD, ORC_HARDSHRINK, ORC_SOFTSHRINK, ORC_LOGIT,
       ORC_NAN_TO_NUM, ORC_ROUND_DECIMALS, ORC_GELU_TANH };
enum { ORC_ADDCMUL = 0, ORC_ADDCDIV, ORC_LERP };
enum { ORC_SUM = 0, ORC_MEAN, ORC_AMAX, ORC_ARGMAX, ORC_PROD, ORC_VAR, ORC_AMIN, ORC_ARGMIN, ORC_STD, ORC_ANY, ORC_ALL,
       ORC_LOGSUMEXP, ORC_NANSUM, ORC_NANMEAN, ORC_COUNT_NONZERO, ORC_NORM };

}  // extern "C"

namespace {

// ---------------------------------------------------------------------------
// dtype helpers
// ---------------------------------------------------------------------------
inline int esize(int dt) {
  switch (dt) {
    case ORC_BOOL: return 1;
    case ORC_I32: return 4;
    case ORC_I64: return 8;
    case ORC_F16: return 2;
    case ORC_BF16: return 2;
    case ORC_F32: return 4;
  }
  return 0;
}
inline bool valid_dtype(int dt) { return dt >= ORC_BOOL && dt <= ORC_F32; }
// category: 0 bool, 1 integer, 2 floating
inline int category(int dt) { return dt == ORC_BOOL ? 0 : (dt <= ORC_I64 ? 1 : 2); }
inline bool is_float(int dt) { return category(dt) == 2; }

// Same-rank promotion of two dtypes: within a category the wider type wins,
// fp16 with bf16 gives fp32; across categories the higher category's type is
// kept unchanged.
int promote2(int a, int b) {
  if (a == b) return a;
  int ca = category(a), cb = category(b);
  if (ca != cb) return ca > cb ? a : b;
  if (ca == 1) return ORC_I64;                       // int32 with int64
  // two different floating types
  if (a == ORC_F32 || b == ORC_F32) return ORC_F32;
  return ORC_F32;                                    // fp16 with bf16
}

// Result dtype of an n-ary tensor op.  Dimensioned operands (ndim >= 1) and
// 0-dim operands are promoted as two separate groups; the 0-dim group changes
// the result only when it is of a strictly higher category.
int result_type(const orc_tensor* const* ops, int n) {
  int D = -1, Z = -1;
  for (int i = 0; i < n; ++i) {
    if (ops[i]->ndim >= 1) D = D < 0 ? ops[i]->dtype : promote2(D, ops[i]->dtype);
    else                   Z = Z < 0 ? ops[i]->dtype : promote2(Z, ops[i]->dtype);
  }
  if (D < 0) return Z;
  if (Z < 0) return D;
  return category(D) >= category(Z) ? D : Z;
}

// ---------------------------------------------------------------------------
// binary16 / bfloat16 encodings, written from the IEEE-754 format definition.
// ---------------------------------------------------------------------------
// Decode a small binary format with `mb` mantissa bits and `eb` exponent bits.
double decode_small(uint32_t bits, int eb, int mb) {
  uint32_t sign = (bits >> (eb + mb)) & 1u;
  uint32_t e = (bits >> mb) & ((1u << eb) - 1u);
  uint32_t m = bits & ((1u << mb) - 1u);
  int bias = (1 << (eb - 1)) - 1;
  double v;
  if (e == (1u << eb) - 1u) {
    v = m ? std::numeric_limits<double>::quiet_NaN() : std::numeric_limits<double>::infinity();
  } else if (e == 0) {
    v = std::ldexp((double)m, 1 - bias - mb);        // subnormal (or zero)
  } else {
    v = std::ldexp((double)((1u << mb) | m), (int)e - bias - mb);
  }
  return sign ? -v : v;
}

// Round a binary64 value once (nearest, ties to even) into the small format.
uint32_t encode_small(double v, int eb, int mb) {
  uint32_t signbit = std::signbit(v) ? (1u << (eb + mb)) : 0u;
  uint32_t emax_field = (1u << eb) - 1u;
  int bias = (1 << (eb - 1)) - 1;
  if (std::isnan(v)) return signbit | (emax_field << mb) | (1u << (mb - 1));
  double a = std::fabs(v);
  if (std::isinf(a)) return signbit | (emax_field << mb);
  if (a == 0.0) return signbit;
  int e;
  std::frexp(a, &e);                                 // a = f * 2^e, f in [0.5,1)
  int E = e - 1;                                     // a = 1.xxx * 2^E
  int emin = 1 - bias;
  if (E < emin) E = emin;                            // subnormal quantum
  // a / 2^(E-mb) is an exact scaling; nearbyint rounds half to even in the
  // default rounding mode.
  double q = std::nearbyint(std::ldexp(a, -(E - mb)));
  // q is in [0, 2^(mb+1)]; renormalise if rounding carried out.
  if (q >= std::ldexp(1.0, mb + 1)) { q = std::ldexp(q, -1); E += 1; }
  if (E > bias) return signbit | (emax_field << mb);  // overflow to infinity
  uint64_t qi = (uint64_t)q;
  if (qi < (1ull << mb)) {
    // subnormal (E == emin and no hidden bit) or zero
    return signbit | (uint32_t)qi;
  }
  uint32_t efield = (uint32_t)(E + bias);
  return signbit | (efield << mb) | (uint32_t)(qi & ((1ull << mb) - 1ull));
}

inline double f16_to_double(uint16_t h) { return decode_small(h, 5, 10); }
inline double bf16_to_double(uint16_t h) { return decode_small(h, 8, 7); }
inline uint16_t double_to_f16(double v) { return (uint16_t)encode_small(v, 5, 10); }
inline uint16_t double_to_bf16(double v) { return (uint16_t)encode_small(v, 8, 7); }

// ---------------------------------------------------------------------------
// typed element access
// ---------------------------------------------------------------------------
inline const char* cptr(const orc_tensor* t, int64_t off) {
  return (const char*)t->data + off * esize(t->dtype);
}
inline char* mptr(const orc_tensor* t, int64_t off) {
  return (char*)t->data + off * esize(t->dtype);
}

// integer-valued read (bool, int32, int64)
inline int64_t load_int(const orc_tensor* t, int64_t off) {
  const char* p = cptr(t, off);
  switch (t->dtype) {
    case ORC_BOOL: { uint8_t v; std::memcpy(&v, p, 1); return v != 0; }
    case ORC_I32: { int32_t v; std::memcpy(&v, p, 4); return v; }
    case ORC_I64: { int64_t v; std::memcpy(&v, p, 8); return v; }
  }
  return 0;
}
// floating read, exact (fp16, bf16, fp32 are all exactly representable)
inline double load_flt(const orc_tensor* t, int64_t off) {
  const char* p = cptr(t, off);
  switch (t->dtype) {
    case ORC_F16: { uint16_t v; std::memcpy(&v, p, 2); return f16_to_double(v); }
    case ORC_BF16: { uint16_t v; std::memcpy(&v, p, 2); return bf16_to_double(v); }
    case ORC_F32: { float v; std::memcpy(&v, p, 4); return (double)v; }
  }
  return 0.0;
}

// A value in some "common dtype": integers/bools live in `i`, floats in `f`.
// For a floating common dtype the value held is already rounded to that dtype.
struct Val {
  int64_t i;
  float f;
};

inline float round_to_float_dtype(double v, int dt) {
  switch (dt) {
    case ORC_F16: return (float)f16_to_double(double_to_f16(v));
    case ORC_BF16: return (float)bf16_to_double(double_to_bf16(v));
    default: return (float)v;
  }
}

// Read operand element and convert it to the common dtype `cd`.
inline Val load_as(const orc_tensor* t, int64_t off, int cd) {
  Val r{0, 0.0f};
  if (is_float(t->dtype)) {
    double v = load_flt(t, off);
    // a float operand is only ever converted to another float dtype here
    r.f = (t->dtype == cd) ? (float)v : round_to_float_dtype(v, cd);
    return r;
  }
  int64_t v = load_int(t, off);
  switch (cd) {
    case ORC_BOOL: r.i = v != 0; break;
    case ORC_I32: r.i = (int64_t)(int32_t)(uint32_t)(uint64_t)v; break;
    case ORC_I64: r.i = v; break;
    case ORC_F32: r.f = (float)v; break;              // nearest-even
    default: r.f = round_to_float_dtype((double)v, cd); break;
  }
  return r;
}

inline void store_int(const orc_tensor* t, int64_t off, int64_t v) {
  char* p = mptr(t, off);
  switch (t->dtype) {
    case ORC_BOOL: { uint8_t b = v != 0; std::memcpy(p, &b, 1); break; }
    case ORC_I32: { int32_t w = (int32_t)(uint32_t)(uint64_t)v; std::memcpy(p, &w, 4); break; }
    case ORC_I64: std::memcpy(p, &v, 8); break;
  }
}
// one rounding from binary64 into the floating output dtype
inline void store_flt(const orc_tensor* t, int64_t off, double v) {
  char* p = mptr(t, off);
  switch (t->dtype) {
    case ORC_F16: { uint16_t h = double_to_f16(v); std::memcpy(p, &h, 2); break; }
    case ORC_BF16: { uint16_t h = double_to_bf16(v); std::memcpy(p, &h, 2); break; }
    case ORC_F32: { float f = (float)v; std::memcpy(p, &f, 4); break; }
  }
}

// `out=` casting.  An operator's result is formed in its result dtype `rd` and then converted to the dtype of
// the tensor it is written to; the conversion must not lose the value's kind: a floating result cannot go to an
// integer or bool tensor, an integer result cannot go to a bool tensor, everything else is allowed.
inline bool can_cast(int from, int to) {
  if (is_float(from) && !is_float(to)) return false;
  if (from != ORC_BOOL && to == ORC_BOOL) return false;
  return true;
}
// floating result: round to rd (once, from binary64), then to out's dtype (exact when out is wider)
inline void put_flt(const orc_tensor* out, int64_t off, int rd, double v) {
  store_flt(out, off, out->dtype == rd ? v : (double)round_to_float_dtype(v, rd));
}
// integer / bool result: wrap to rd, then convert; an integer goes to a floating dtype through binary32
inline void put_int(const orc_tensor* out, int64_t off, int rd, int64_t v) {
  int64_t w = rd == ORC_BOOL ? (int64_t)(v != 0) : rd == ORC_I32 ? (int64_t)(int32_t)(uint32_t)(uint64_t)v : v;
  if (is_float(out->dtype)) store_flt(out, off, (double)(float)w);
  else store_int(out, off, w);
}

// ---------------------------------------------------------------------------
// shapes
// ---------------------------------------------------------------------------
inline int64_t numel(const orc_tensor* t) {
  int64_t n = 1;
  for (int d = 0; d < t->ndim; ++d) n *= t->sizes[d];
  return n;
}
int check_tensor(const orc_tensor* t) {
  if (!t) return ORC_ERR_NULL;
  if (t->ndim < 0 || t->ndim > ORC_MAX_DIMS) return ORC_ERR_NDIM;
  if (!valid_dtype(t->dtype)) return ORC_ERR_DTYPE;
  for (int d = 0; d < t->ndim; ++d)
    if (t->sizes[d] < 0) return ORC_ERR_SHAPE;
  if (numel(t) > 0 && !t->data) return ORC_ERR_NULL;
  return ORC_OK;
}

// Broadcast a list of shapes (right-aligned).  Returns <0 if incompatible.
int broadcast_shapes(const orc_tensor* const* ops, int n, int* ondim, int64_t* osizes) {
  int nd = 0;
  for (int i = 0; i < n; ++i) nd = std::max(nd, (int)ops[i]->ndim);
  for (int d = 0; d < nd; ++d) osizes[d] = 1;
  for (int i = 0; i < n; ++i) {
    int shift = nd - ops[i]->ndim;
    for (int d = 0; d < ops[i]->ndim; ++d) {
      int64_t s = ops[i]->sizes[d];
      int64_t& o = osizes[d + shift];
      if (s == o) continue;
      if (o == 1) o = s;
      else if (s != 1) return ORC_ERR_SHAPE;
    }
  }
  *ondim = nd;
  return ORC_OK;
}

// Turn a linear logical (row-major) index over `sizes` into a multi-index.
inline void unravel(int64_t lin, int nd, const int64_t* sizes, int64_t* idx) {
  for (int d = nd - 1; d >= 0; --d) {
    int64_t s = sizes[d];
    idx[d] = s ? lin % s : 0;
    lin = s ? lin / s : 0;
  }
}
inline int64_t offset_of(const orc_tensor* t, const int64_t* idx) {
  int64_t o = 0;
  for (int d = 0; d < t->ndim; ++d) o += idx[d] * t->strides[d];
  return o;
}
// offset of operand `t` for output multi-index `idx` of rank `nd`, with
// broadcasting: right-aligned, size-1 dims of the operand do not move.
inline int64_t bcast_offset(const orc_tensor* t, int nd, const int64_t* idx) {
  int shift = nd - t->ndim;
  int64_t o = 0;
  for (int d = 0; d < t->ndim; ++d)
    if (t->sizes[d] != 1) o += idx[d + shift] * t->strides[d];
  return o;
}
bool same_shape(const orc_tensor* t, int nd, const int64_t* sizes) {
  if (t->ndim != nd) return false;
  for (int d = 0; d < nd; ++d)
    if (t->sizes[d] != sizes[d]) return false;
  return true;
}

// integer power with wrapping multiplication: the product of e copies of b, written as the plain loop for small
// e and by squaring for large e (the two agree modulo 2^64); negative e is the truncated reciprocal
int64_t int_pow(int64_t b, int64_t e) {
  if (e < 0) {
    if (b == 1) return 1;
    if (b == -1) return (e % 2 != 0) ? -1 : 1;
    return 0;
  }
  uint64_t r = 1, m = (uint64_t)b;
  for (uint64_t k = (uint64_t)e; k; k >>= 1) {
    if (k & 1) r *= m;
    m *= m;
  }
  return (int64_t)r;
}

// greatest common divisor of the magnitudes (Euclid); gcd(0, 0) = 0
// Floor of a / b in binary32: (a - fmod(a, b)) / b is an integer up to rounding; one is subtracted when the remainder
// and the divisor differ in sign, the result is snapped to the integer next to it, a zero takes the quotient's sign,
// and a zero divisor gives the IEEE quotient (an infinity or NaN).
static float floor_quotient(float a, float b) {
  if (b == 0.0f) return a / b;
  const float mod = std::fmod(a, b);
  float div = (a - mod) / b;
  if (mod != 0.0f && ((b < 0.0f) != (mod < 0.0f))) div -= 1.0f;
  if (div == 0.0f) return std::copysign(0.0f, a / b);
  float fl = std::floor(div);
  if (div - fl > 0.5f) fl += 1.0f;
  return fl;
}
uint64_t gcd_mag(int64_t a, int64_t b) {
  uint64_t x = a < 0 ? 0 - (uint64_t)a : (uint64_t)a, y = b < 0 ? 0 - (uint64_t)b : (uint64_t)b;
  while (y) {
    uint64_t t = x % y;
    x = y;
    y = t;
  }
  return x;
}

// the value of format `dt` next to a in the direction of b: b when they are equal, the smallest subnormal when a
// is a zero, otherwise one step on a's encoding (sign-magnitude, so magnitude + 1 moves away from zero and the
// largest finite value steps to infinity); NaN when either is NaN
double next_toward(double a, double b, int dt) {
  if (std::isnan(a) || std::isnan(b)) return std::numeric_limits<double>::quiet_NaN();
  if (a == b) return b;
  const bool away = (a < b) == (a > 0.0);           // the step grows the magnitude
  if (dt == ORC_F32) {
    uint32_t u;
    float f = (float)a;
    if (a == 0.0) { u = (b < 0.0 ? 0x80000000u : 0u) | 1u; }
    else { std::memcpy(&u, &f, 4); u = away ? u + 1 : u - 1; }
    std::memcpy(&f, &u, 4);
    return (double)f;
  }
  uint16_t h;
  if (a == 0.0) h = (uint16_t)((b < 0.0 ? 0x8000u : 0u) | 1u);
  else {
    h = dt == ORC_F16 ? double_to_f16(a) : double_to_bf16(a);
    h = (uint16_t)(away ? h + 1 : h - 1);
  }
  return dt == ORC_F16 ? f16_to_double(h) : bf16_to_double(h);
}

const double kNaN = std::numeric_limits<double>::quiet_NaN();
const double kInf = std::numeric_limits<double>::infinity();

}  // namespace

extern "C" {

// ===========================================================================
// Result inference (dtype and shape), usable without data pointers.
// ===========================================================================

// Result dtype of a unary op given the input dtype, or an error.
int orc_unary_result_dtype(int op, int in_dtype) {
  if (!valid_dtype(in_dtype)) return ORC_ERR_DTYPE;
  switch (op) {
    case ORC_NEG:
    case ORC_ABS:
      return in_dtype == ORC_BOOL ? ORC_ERR_DTYPE : in_dtype;
    case ORC_EXP: case ORC_LOG: case ORC_SQRT: case ORC_SIGMOID: case ORC_TANH: case ORC_LOG1P: case ORC_EXPM1:
      return is_float(in_dtype) ? in_dtype : ORC_F32;   // integral input computes in fp32
    case ORC_GELU: case ORC_LOGSIGMOID:
      return is_float(in_dtype) ? in_dtype : ORC_ERR_DTYPE;
    case ORC_LOGICAL_NOT: case ORC_ISNAN: case ORC_ISINF: case ORC_ISFINITE:
      return ORC_BOOL;
    case ORC_SIN: case ORC_COS: case ORC_EXP2: case ORC_LOG2: case ORC_LOG10: case ORC_RSQRT: case ORC_RECIPROCAL:
      return is_float(in_dtype) ? in_dtype : ORC_F32;
    case ORC_SILU:
      return is_float(in_dtype) ? in_dtype : ORC_ERR_DTYPE;
    case ORC_SQUARE:
      return in_dtype == ORC_BOOL ? ORC_I64 : in_dtype;    // a bool squares as the integer 0 / 1
    case ORC_SIGN:
      return in_dtype;
    case ORC_FLOOR: case ORC_CEIL: case ORC_TRUNC: case ORC_ROUND:
      return in_dtype == ORC_BOOL ? ORC_ERR_DTYPE : in_dtype;
    case ORC_BITWISE_NOT:
      return is_float(in_dtype) ? ORC_ERR_DTYPE : in_dtype;
    case ORC_TAN: case ORC_ASIN: case ORC_ACOS: case ORC_ATAN: case ORC_SINH: case ORC_COSH: case ORC_ASINH: case ORC_ACOSH:
    case ORC_ATANH: case ORC_ERF: case ORC_ERFC:
      return is_float(in_dtype) ? in_dtype : ORC_F32;
    case ORC_RELU:
      return in_dtype == ORC_BOOL ? ORC_ERR_DTYPE : in_dtype;
    case ORC_FRAC: case ORC_HARDSWISH: case ORC_HARDSIGMOID: case ORC_MISH:
      return is_float(in_dtype) ? in_dtype : ORC_ERR_DTYPE;
    case ORC_SIGNBIT:
      return ORC_BOOL;
  }
  return ORC_ERR_DTYPE;
}

// Result dtype + broadcast shape of a binary op (ADD MUL DIV MAXIMUM EQ).
int orc_infer_binary(int op, const orc_tensor* a, const orc_tensor* b, int32_t* dtype, int32_t* ndim,
                     int64_t* sizes) {
  if (!a || !b) return ORC_ERR_NULL;
  if (!valid_dtype(a->dtype) || !valid_dtype(b->dtype)) return ORC_ERR_DTYPE;
  if (a->ndim < 0 || a->ndim > ORC_MAX_DIMS || b->ndim < 0 || b->ndim > ORC_MAX_DIMS) return ORC_ERR_NDIM;
  const orc_tensor* ops[2] = {a, b};
  int common = result_type(ops, 2);
  int res = common;
  if (op < ORC_ADD || op > ORC_TRUNC_DIVIDE) return ORC_ERR_DTYPE;
  if (op == ORC_DIV && !is_float(common)) res = ORC_F32;   // true division
  if (op == ORC_EQ || (op >= ORC_NE && op <= ORC_LOGICAL_XOR)) res = ORC_BOOL;   // comparison and logical families
  if (op == ORC_POW && common == ORC_BOOL) return ORC_ERR_DTYPE;                 // no bool power
  if (op >= ORC_BITWISE_AND && op <= ORC_BITWISE_XOR && is_float(common)) return ORC_ERR_DTYPE;
  if (op == ORC_ATAN2 && !is_float(common)) res = ORC_F32;
  if ((op == ORC_FMOD || op == ORC_REMAINDER || op == ORC_FLOOR_DIVIDE || op == ORC_TRUNC_DIVIDE) && common == ORC_BOOL) return ORC_ERR_DTYPE;
  if ((op == ORC_HYPOT || op == ORC_LOGADDEXP || op == ORC_LOGADDEXP2 || op == ORC_NEXTAFTER) && !is_float(common)) return ORC_ERR_DTYPE;
  if ((op == ORC_COPYSIGN || op == ORC_XLOGY) && !is_float(common)) res = ORC_F32;
  if (op == ORC_HEAVISIDE && a->dtype != b->dtype) return ORC_ERR_DTYPE;        // no promotion between the two
  if (op >= ORC_GCD && op <= ORC_SHIFT_RIGHT && (is_float(common) || common == ORC_BOOL)) return ORC_ERR_DTYPE;
  if (op == ORC_SUB && (a->dtype == ORC_BOOL || b->dtype == ORC_BOOL)) return ORC_ERR_DTYPE;   // no bool subtraction
  int nd;
  int64_t s[ORC_MAX_DIMS];
  int rc = broadcast_shapes(ops, 2, &nd, s);
  if (rc) return rc;
  if (dtype) *dtype = res;
  if (ndim) *ndim = nd;
  if (sizes) for (int d = 0; d < nd; ++d) sizes[d] = s[d];
  return ORC_OK;
}

// Result dtype of where(cond, x, y): promotion of x and y only.
int orc_where_result_dtype(const orc_tensor* x, const orc_tensor* y) {
  const orc_tensor* ops[2] = {x, y};
  return result_type(ops, 2);
}

// ===========================================================================
// Elementwise: unary
// ===========================================================================
// out[i] = f(a[i]).  `out` must have a's shape; its dtype is the inferred one or any dtype that one can be cast to
// (see can_cast): the result is rounded to the inferred dtype first, then converted.
//   logical_not   : x == 0 for any dtype, bool result.
//   sin cos exp2 log2 log10 rsqrt reciprocal : like exp (binary64 evaluation, bool / integer input computes in fp32);
//                   rsqrt = 1 / sqrt(x).  silu = x / (1 + exp(-x)), floating dtypes only.
//   square        : x * x (integers wrap; a bool gives the int64 0 / 1).  sign: -1, 0, 1 in the input's dtype, 0 for
//                   a NaN and for -0.0 (the value of (0 < x) - (x < 0)); a bool is returned as it is.
//   floor ceil trunc round : floats (round: halves to even, the sign of zero is kept); integers are returned as they
//                   are; bool is a dtype error.  isnan / isinf / isfinite: bool result, integers are finite.
//   bitwise_not   : ~x for integers, logical not for bool, floats are a dtype error.
//   tan asin acos atan sinh cosh asinh acosh atanh erf erfc : like exp.
//   relu          : x < 0 ? 0 : x (a NaN and -0.0 stay); integers too; bool is a dtype error.
//   frac          : x - trunc(x) (so frac(+-inf) is NaN); hardsigmoid: min(max(x + 3, 0), 6) / 6; hardswish: x times
//                   that; mish: x * tanh(log1p(exp(x))).  Floating dtypes only; a NaN gives NaN.
//   signbit       : the sign bit of a float (-0.0 and negative NaNs included), x < 0 for an integer, false for a bool.
//   neg, abs      : exact; integers wrap (abs(INT_MIN) == INT_MIN); floats
//                   flip / clear the sign bit (NaN and zeros included).
//   exp log sqrt sigmoid tanh : binary64 evaluation of the input converted to
//                   the result dtype, one rounding.  sigmoid = 1/(1+exp(-x)).
//   gelu (erf form) : x * Phi(x), Phi the standard normal CDF.  Phi is taken
//                   as erfc(-x/sqrt 2)/2, which is the same function as
//                   (1+erf(x/sqrt 2))/2 but keeps its relative accuracy in the
//                   negative tail, so the value rounded here is the true one.
int orc_unary(int op, const orc_tensor* out, const orc_tensor* a) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(a))) return rc;
  int rd = orc_unary_result_dtype(op, a->dtype);
  if (rd < 0) return rd;
  if (!can_cast(rd, out->dtype)) return ORC_ERR_DTYPE;
  if (!same_shape(out, a->ndim, a->sizes)) return ORC_ERR_SHAPE;
  const int64_t n = numel(out);
  const int nd = a->ndim;
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, out->sizes, idx);
    int64_t oo = offset_of(out, idx), ao = offset_of(a, idx);
    if (op == ORC_LOGICAL_NOT) {                      // x == 0 (a NaN is not zero)
      bool zero = is_float(a->dtype) ? load_flt(a, ao) == 0.0 : load_int(a, ao) == 0;
      put_int(out, oo, ORC_BOOL, zero);
      continue;
    }
    if (op == ORC_NEG || op == ORC_ABS) {
      if (is_float(rd)) {
        // sign-bit operations on the stored encoding: exact for every input
        int es = esize(rd);
        uint32_t bits = 0;
        std::memcpy(&bits, cptr(a, ao), es);
        uint32_t sb = 1u << (8 * es - 1);
        bits = (op == ORC_NEG) ? (bits ^ sb) : (bits & ~sb);
        if (out->dtype == rd) {
          std::memcpy(mptr(out, oo), &bits, es);
        } else {                                      // out= casting: the value, converted
          double v = rd == ORC_F16 ? f16_to_double((uint16_t)bits) : rd == ORC_BF16 ? bf16_to_double((uint16_t)bits) : 0.0;
          if (rd == ORC_F32) { float f; std::memcpy(&f, &bits, 4); v = (double)f; }
          store_flt(out, oo, v);
        }
      } else {
        int64_t v = load_int(a, ao);
        uint64_t u = (uint64_t)v;
        if (op == ORC_NEG) u = 0 - u;
        else if (v < 0) u = 0 - u;
        put_int(out, oo, rd, (int64_t)u);             // wraps to the result dtype
      }
      continue;
    }
    if (op == ORC_SIGNBIT) {
      bool neg;
      if (is_float(a->dtype)) {
        const int es = esize(a->dtype);
        uint32_t bits = 0;
        std::memcpy(&bits, cptr(a, ao), es);
        neg = (bits >> (8 * es - 1)) & 1u;
      } else {
        neg = a->dtype != ORC_BOOL && load_int(a, ao) < 0;
      }
      put_int(out, oo, ORC_BOOL, neg);
      continue;
    }
    if (op == ORC_RELU && !is_float(a->dtype)) {
      const int64_t v = load_int(a, ao);
      put_int(out, oo, rd, v < 0 ? 0 : v);
      continue;
    }
    if (op == ORC_ISNAN || op == ORC_ISINF || op == ORC_ISFINITE) {       // integers and bools are always finite
      const double v = is_float(a->dtype) ? load_flt(a, ao) : 0.0;
      put_int(out, oo, ORC_BOOL, op == ORC_ISNAN ? std::isnan(v) : op == ORC_ISINF ? std::isinf(v) : std::isfinite(v));
      continue;
    }
    if (!is_float(a->dtype) && (op == ORC_SQUARE || op == ORC_SIGN || op == ORC_FLOOR || op == ORC_CEIL || op == ORC_TRUNC ||
                                op == ORC_ROUND || op == ORC_BITWISE_NOT)) {
      const int64_t v = load_int(a, ao);
      int64_t r = v;                                  // floor / ceil / trunc / round of an integer: itself
      if (op == ORC_SQUARE) r = (int64_t)((uint64_t)v * (uint64_t)v);
      else if (op == ORC_SIGN) r = (v > 0) - (v < 0);
      else if (op == ORC_BITWISE_NOT) r = a->dtype == ORC_BOOL ? !v : ~v;
      put_int(out, oo, rd, r);
      continue;
    }
    double x = (double)load_as(a, ao, rd).f;          // converted to result dtype first
    double y = 0.0;
    switch (op) {
      case ORC_SIN: y = std::sin(x); break;
      case ORC_COS: y = std::cos(x); break;
      case ORC_EXP2: y = std::exp2(x); break;
      case ORC_LOG2: y = std::log2(x); break;
      case ORC_LOG10: y = std::log10(x); break;
      case ORC_RSQRT: y = 1.0 / std::sqrt(x); break;
      case ORC_RECIPROCAL: y = 1.0 / x; break;
      case ORC_SILU: y = x / (1.0 + std::exp(-x)); break;                // x * sigmoid(x)
      case ORC_SQUARE: y = x * x; break;                                   // exact in binary64, one rounding on store
      case ORC_SIGN: y = (double)((0.0 < x) - (x < 0.0)); break;          // 0 for a NaN and for either zero
      case ORC_FLOOR: y = std::floor(x); break;
      case ORC_CEIL: y = std::ceil(x); break;
      case ORC_TRUNC: y = std::trunc(x); break;
      case ORC_ROUND: y = std::nearbyint(x); break;                        // halves to even (default rounding mode)
      case ORC_EXP: y = std::exp(x); break;
      case ORC_LOG: y = std::log(x); break;
      case ORC_SQRT: y = std::sqrt(x); break;
      case ORC_SIGMOID: y = 1.0 / (1.0 + std::exp(-x)); break;
      case ORC_TANH: y = std::tanh(x); break;
      case ORC_GELU: y = x * (0.5 * std::erfc(-x * 0.70710678118654752440)); break;
      case ORC_LOG1P: y = std::log1p(x); break;
      case ORC_EXPM1: y = std::expm1(x); break;
      // log(1 / (1 + exp(-x))) written so that neither tail overflows or cancels: min(x, 0) - log1p(exp(-|x|))
      case ORC_LOGSIGMOID: y = (x < 0.0 ? x : 0.0) - std::log1p(std::exp(-std::fabs(x))); break;
      case ORC_TAN: y = std::tan(x); break;
      case ORC_ASIN: y = std::asin(x); break;
      case ORC_ACOS: y = std::acos(x); break;
      case ORC_ATAN: y = std::atan(x); break;
      case ORC_SINH: y = std::sinh(x); break;
      case ORC_COSH: y = std::cosh(x); break;
      case ORC_ASINH: y = std::asinh(x); break;
      case ORC_ACOSH: y = std::acosh(x); break;
      case ORC_ATANH: y = std::atanh(x); break;
      case ORC_ERF: y = std::erf(x); break;
      case ORC_ERFC: y = std::erfc(x); break;
      case ORC_RELU: y = x < 0.0 ? 0.0 : x; break;
      case ORC_FRAC: y = x - std::trunc(x); break;
      case ORC_HARDSIGMOID: case ORC_HARDSWISH: {
        double t = x + 3.0;
        t = t < 0.0 ? 0.0 : t;                      // a NaN fails both comparisons and stays
        t = t > 6.0 ? 6.0 : t;
        y = op == ORC_HARDSWISH ? x * t / 6.0 : t / 6.0;
        break;
      }
      case ORC_MISH: y = x * std::tanh(std::log1p(std::exp(x))); break;
    }
    put_flt(out, oo, rd, y);
  }
  return ORC_OK;
}

// ===========================================================================
// Elementwise: binary with broadcasting and type promotion
// ===========================================================================
// out = a (op) b on the broadcast shape.  Both operands are converted to the
// common dtype first, then the op is applied.
//   add     : a + alpha*b.  bool: a OR (alpha!=0 AND b).  integers: wrapping,
//             alpha must be integral.  floats: alpha==1 is a single IEEE add;
//             alpha!=1 is a single-rounding fused multiply-add fma(alpha,b,a)
//             in binary32 (the half types compute in binary32 and round).
//   mul     : product; bool AND; integers wrap.
//   div     : true division; bool/integer operands are converted to fp32.
//   maximum : NaN if either operand is NaN, else the larger (first operand on
//             ties).
//   eq      : equality in the common dtype, bool result.
//   sub     : a - alpha*b with the rules of add (one IEEE subtraction, or one
//             fma(-alpha, b, a)); any bool operand is a dtype error.
//   minimum : NaN if either operand is NaN, else the smaller (first operand on
//             ties); bool AND.
//   ne lt le gt ge : IEEE comparisons in the common dtype, bool result (every
//             ordered comparison with a NaN is false, ne is true).
//   logical_and / or / xor : (a != 0) op (b != 0) in the common dtype, bool
//             result; a NaN counts as non-zero.
//   pow     : a to the power b.  Floating common dtype: the binary64 power of
//             the converted operands (C Annex F special values: anything^0 = 1,
//             1^anything = 1, negative base with a non-integer exponent = NaN,
//             ...), one rounding.  Integer common dtype: wrapping product of b
//             copies of a; for b < 0 the truncated reciprocal: 1 for a == 1,
//             +-1 for a == -1 by b's parity, 0 otherwise (0^negative included).
//             Two bool operands are a dtype error.
//   bitwise_and / or / xor : on the two's-complement integers of the common
//             dtype (bool: the logical operation); a floating common dtype is
//             a dtype error.
//   atan2   : the angle of the point (b, a), binary64 evaluation of the
//             converted operands, one rounding; bool / integer operands are
//             converted to fp32.
//   fmod    : the remainder with the dividend's sign (C fmod / integer %);
//             remainder: the one with the divisor's sign (fmod, plus the
//             divisor when the signs differ and the value is not zero).
//             bool is a dtype error; an integer zero divisor is ORC_ERR_SCALAR.
//   floor_divide / trunc_divide (ATen's div with rounding_mode "floor" / "trunc"): the quotient rounded toward
//             -infinity / toward zero, in the common dtype (integers stay integers; int32 wraps; bool is a dtype
//             error; an integer zero divisor is ORC_ERR_SCALAR).  Floating operands follow ATen in binary32
//             (bf16 / fp16 operands converted first): trunc truncates the quotient after it has been rounded to the
//             common format, as ATen does on every device (5.99 / 1 in bf16 is 6, not 5); floor is
//             floor_quotient() above, rounded to the common format once at the end, the algorithm ATen shares with Python's float floor
//             division, which starts from the exact fmod so that a quotient just below an integer is not
//             rounded up to it by the division.
//   hypot   : sqrt(a^2 + b^2) without intermediate overflow, +inf when either
//             is infinite; logaddexp: log(e^a + e^b) as max + log1p(exp(-|a-b|)),
//             equal infinities give themselves; logaddexp2: the base-2 form;
//             nextafter: the neighbour of a toward b in the common format.
//             Floating common dtype only.
//   copysign: |a| with b's sign bit; xlogy: NaN if b is NaN, else 0 if a == 0,
//             else a * log(b).  bool / integer operands are converted to fp32.
//   heaviside: 0 for a < 0 and for a NaN a, 1 for a > 0, b for a == 0; both
//             operands must have the same dtype.
//   fmax / fmin : the larger / smaller; a NaN only when both are NaN.
//   gcd / lcm : of the magnitudes, wrapped to the dtype (gcd(0,0) = lcm(0,x) =
//             0); shift_left / shift_right: a << b and the arithmetic a >> b; a
//             shift count below 0 or at least the width gives 0, or -1 for a
//             negative a shifted right.  int32 / int64 only.
// `out` may have any dtype the result dtype can be cast to (can_cast): the
// value is formed in the result dtype, then converted.
int orc_binary(int op, const orc_tensor* out, const orc_tensor* a, const orc_tensor* b, double alpha_f,
               int64_t alpha_i, int alpha_is_int) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(a)) || (rc = check_tensor(b))) return rc;
  int32_t rd, nd;
  int64_t sizes[ORC_MAX_DIMS];
  if ((rc = orc_infer_binary(op, a, b, &rd, &nd, sizes))) return rc;
  if (!can_cast(rd, out->dtype)) return ORC_ERR_DTYPE;
  if (!same_shape(out, nd, sizes)) return ORC_ERR_SHAPE;
  const orc_tensor* ops[2] = {a, b};
  int cd = result_type(ops, 2);                       // dtype the op is applied in
  if ((op == ORC_DIV || op == ORC_ATAN2 || op == ORC_COPYSIGN || op == ORC_XLOGY) && !is_float(cd)) cd = ORC_F32;
  if ((op == ORC_ADD || op == ORC_SUB) && !is_float(cd) && !alpha_is_int) return ORC_ERR_SCALAR;
  const double alpha_d = alpha_is_int ? (double)alpha_i : alpha_f;
  const float alpha32 = (float)alpha_d;
  const bool alpha_one = alpha_is_int ? (alpha_i == 1) : (alpha_f == 1.0);
  const int64_t n = numel(out);
  if ((op == ORC_FMOD || op == ORC_REMAINDER || op == ORC_FLOOR_DIVIDE || op == ORC_TRUNC_DIVIDE) && !is_float(cd))   // an integer zero divisor anywhere: nothing is written
    for (int64_t lin = 0; lin < n; ++lin) {
      int64_t idx[ORC_MAX_DIMS];
      unravel(lin, nd, sizes, idx);
      if (load_as(b, bcast_offset(b, nd, idx), cd).i == 0) return ORC_ERR_SCALAR;
    }
  const int width = cd == ORC_I32 ? 32 : 64;
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, sizes, idx);
    int64_t oo = offset_of(out, idx);
    Val x = load_as(a, bcast_offset(a, nd, idx), cd);
    Val y = load_as(b, bcast_offset(b, nd, idx), cd);
    if (is_float(cd)) {
      const double xd = (double)x.f, yd = (double)y.f;
      switch (op) {
        case ORC_FMOD: put_flt(out, oo, rd, std::fmod(xd, yd)); break;
        case ORC_REMAINDER: {
          double r = std::fmod(xd, yd);
          if (r != 0.0 && ((r < 0.0) != (yd < 0.0))) r += yd;
          put_flt(out, oo, rd, r);
          break;
        }
        case ORC_TRUNC_DIVIDE:                   // the quotient as the common format holds it, then truncated
          put_flt(out, oo, rd, (double)std::trunc(round_to_float_dtype((double)(x.f / y.f), cd)));
          break;
        case ORC_FLOOR_DIVIDE: put_flt(out, oo, rd, (double)floor_quotient(x.f, y.f)); break;
        case ORC_HYPOT: put_flt(out, oo, rd, std::hypot(xd, yd)); break;
        case ORC_COPYSIGN: put_flt(out, oo, rd, std::copysign(xd, yd)); break;
        case ORC_LOGADDEXP: case ORC_LOGADDEXP2: {
          double r;
          if (std::isnan(xd) || std::isnan(yd)) r = kNaN;
          else if (std::isinf(xd) && xd == yd) r = xd;
          else {
            const double m = xd > yd ? xd : yd, d = -std::fabs(xd - yd);
            r = op == ORC_LOGADDEXP ? m + std::log1p(std::exp(d)) : m + std::log1p(std::exp2(d)) / std::log(2.0);
          }
          put_flt(out, oo, rd, r);
          break;
        }
        case ORC_XLOGY: put_flt(out, oo, rd, std::isnan(yd) ? kNaN : xd == 0.0 ? 0.0 : xd * std::log(yd)); break;
        case ORC_HEAVISIDE: put_flt(out, oo, rd, xd == 0.0 ? yd : (xd > 0.0 ? 1.0 : 0.0)); break;
        case ORC_FMAX: put_flt(out, oo, rd, std::isnan(xd) ? yd : std::isnan(yd) ? xd : (yd > xd ? yd : xd)); break;
        case ORC_FMIN: put_flt(out, oo, rd, std::isnan(xd) ? yd : std::isnan(yd) ? xd : (yd < xd ? yd : xd)); break;
        case ORC_NEXTAFTER: put_flt(out, oo, rd, next_toward(xd, yd, cd)); break;
        default: break;
      }
      switch (op) {
        case ORC_ADD: {
          float r = alpha_one ? (x.f + y.f) : std::fmaf(alpha32, y.f, x.f);
          put_flt(out, oo, rd, (double)r);
          break;
        }
        case ORC_MUL: {
          float r = x.f * y.f;
          put_flt(out, oo, rd, (double)r);
          break;
        }
        case ORC_DIV:
          put_flt(out, oo, rd, (double)x.f / (double)y.f);
          break;
        case ORC_MAXIMUM: {
          float r = (std::isnan(x.f) || std::isnan(y.f)) ? std::numeric_limits<float>::quiet_NaN()
                                                         : (y.f > x.f ? y.f : x.f);
          put_flt(out, oo, rd, (double)r);
          break;
        }
        case ORC_EQ: put_int(out, oo, rd, x.f == y.f); break;
        case ORC_SUB: {                               // a - alpha*b: one IEEE subtraction, or one fma(-alpha, b, a)
          float r = alpha_one ? (x.f - y.f) : std::fmaf(-alpha32, y.f, x.f);
          put_flt(out, oo, rd, (double)r);
          break;
        }
        case ORC_MINIMUM: {
          float r = (std::isnan(x.f) || std::isnan(y.f)) ? std::numeric_limits<float>::quiet_NaN()
                                                         : (y.f < x.f ? y.f : x.f);
          put_flt(out, oo, rd, (double)r);
          break;
        }
        case ORC_NE: put_int(out, oo, rd, x.f != y.f); break;    // IEEE: every ordered comparison with NaN is false,
        case ORC_LT: put_int(out, oo, rd, x.f < y.f); break;     // != is true
        case ORC_LE: put_int(out, oo, rd, x.f <= y.f); break;
        case ORC_GT: put_int(out, oo, rd, x.f > y.f); break;
        case ORC_GE: put_int(out, oo, rd, x.f >= y.f); break;
        case ORC_LOGICAL_AND: put_int(out, oo, rd, (x.f != 0.0f) && (y.f != 0.0f)); break;   // a NaN is not zero
        case ORC_LOGICAL_OR: put_int(out, oo, rd, (x.f != 0.0f) || (y.f != 0.0f)); break;
        case ORC_LOGICAL_XOR: put_int(out, oo, rd, (x.f != 0.0f) != (y.f != 0.0f)); break;
        case ORC_POW: put_flt(out, oo, rd, std::pow((double)x.f, (double)y.f)); break;       // C Annex F special cases
        case ORC_ATAN2: put_flt(out, oo, rd, std::atan2((double)x.f, (double)y.f)); break;
      }
    } else if (cd == ORC_BOOL) {
      switch (op) {
        case ORC_ADD: put_int(out, oo, rd, x.i | ((alpha_i != 0) & y.i)); break;
        case ORC_MUL: put_int(out, oo, rd, x.i & y.i); break;
        case ORC_MAXIMUM: put_int(out, oo, rd, x.i | y.i); break;
        case ORC_EQ: put_int(out, oo, rd, x.i == y.i); break;
        case ORC_MINIMUM: put_int(out, oo, rd, x.i & y.i); break;
        case ORC_NE: put_int(out, oo, rd, x.i != y.i); break;
        case ORC_LT: put_int(out, oo, rd, x.i < y.i); break;
        case ORC_LE: put_int(out, oo, rd, x.i <= y.i); break;
        case ORC_GT: put_int(out, oo, rd, x.i > y.i); break;
        case ORC_GE: put_int(out, oo, rd, x.i >= y.i); break;
        case ORC_LOGICAL_AND: put_int(out, oo, rd, x.i & y.i); break;
        case ORC_LOGICAL_OR: put_int(out, oo, rd, x.i | y.i); break;
        case ORC_LOGICAL_XOR: case ORC_BITWISE_XOR: put_int(out, oo, rd, x.i ^ y.i); break;
        case ORC_BITWISE_AND: put_int(out, oo, rd, x.i & y.i); break;
        case ORC_BITWISE_OR: put_int(out, oo, rd, x.i | y.i); break;
        case ORC_HEAVISIDE: put_int(out, oo, rd, x.i ? 1 : y.i); break;
        case ORC_FMAX: put_int(out, oo, rd, x.i | y.i); break;
        case ORC_FMIN: put_int(out, oo, rd, x.i & y.i); break;
      }
    } else {
      uint64_t ux = (uint64_t)x.i, uy = (uint64_t)y.i;
      switch (op) {
        case ORC_ADD: put_int(out, oo, rd, (int64_t)(ux + (uint64_t)alpha_i * uy)); break;
        case ORC_MUL: put_int(out, oo, rd, (int64_t)(ux * uy)); break;
        case ORC_MAXIMUM: put_int(out, oo, rd, y.i > x.i ? y.i : x.i); break;
        case ORC_EQ: put_int(out, oo, rd, x.i == y.i); break;
        case ORC_SUB: put_int(out, oo, rd, (int64_t)(ux - (uint64_t)alpha_i * uy)); break;
        case ORC_MINIMUM: put_int(out, oo, rd, y.i < x.i ? y.i : x.i); break;
        case ORC_NE: put_int(out, oo, rd, x.i != y.i); break;
        case ORC_LT: put_int(out, oo, rd, x.i < y.i); break;
        case ORC_LE: put_int(out, oo, rd, x.i <= y.i); break;
        case ORC_GT: put_int(out, oo, rd, x.i > y.i); break;
        case ORC_GE: put_int(out, oo, rd, x.i >= y.i); break;
        case ORC_LOGICAL_AND: put_int(out, oo, rd, (x.i != 0) && (y.i != 0)); break;
        case ORC_LOGICAL_OR: put_int(out, oo, rd, (x.i != 0) || (y.i != 0)); break;
        case ORC_LOGICAL_XOR: put_int(out, oo, rd, (x.i != 0) != (y.i != 0)); break;
        case ORC_POW: put_int(out, oo, rd, int_pow(x.i, y.i)); break;
        case ORC_BITWISE_AND: put_int(out, oo, rd, x.i & y.i); break;
        case ORC_BITWISE_OR: put_int(out, oo, rd, x.i | y.i); break;
        case ORC_BITWISE_XOR: put_int(out, oo, rd, x.i ^ y.i); break;
        case ORC_FMOD: case ORC_REMAINDER: {
          int64_t r = y.i == -1 ? 0 : x.i % y.i;     // by -1 everything divides (and INT_MIN % -1 is not a C expression)
          if (op == ORC_REMAINDER && r != 0 && ((r < 0) != (y.i < 0))) r += y.i;
          put_int(out, oo, rd, r);
          break;
        }
        case ORC_FLOOR_DIVIDE: case ORC_TRUNC_DIVIDE: {
          int64_t q;
          if (y.i == -1) q = (int64_t)(0 - (uint64_t)x.i);    // the most negative value wraps onto itself
          else {
            q = x.i / y.i;
            if (op == ORC_FLOOR_DIVIDE && x.i % y.i != 0 && ((x.i < 0) != (y.i < 0))) --q;
          }
          put_int(out, oo, rd, q);
          break;
        }
        case ORC_HEAVISIDE: put_int(out, oo, rd, x.i == 0 ? y.i : (x.i > 0 ? 1 : 0)); break;
        case ORC_FMAX: put_int(out, oo, rd, y.i > x.i ? y.i : x.i); break;
        case ORC_FMIN: put_int(out, oo, rd, y.i < x.i ? y.i : x.i); break;
        case ORC_GCD: put_int(out, oo, rd, (int64_t)gcd_mag(x.i, y.i)); break;
        case ORC_LCM: {
          const uint64_t g = gcd_mag(x.i, y.i);
          const uint64_t ua = x.i < 0 ? 0 - ux : ux, ub = y.i < 0 ? 0 - uy : uy;
          put_int(out, oo, rd, g == 0 ? 0 : (int64_t)(ua / g * ub));
          break;
        }
        case ORC_SHIFT_LEFT:
          put_int(out, oo, rd, (y.i < 0 || y.i >= width) ? 0 : (int64_t)(ux << y.i));
          break;
        case ORC_SHIFT_RIGHT:                          // arithmetic: the sign fills
          put_int(out, oo, rd, (y.i < 0 || y.i >= width) ? (x.i < 0 ? -1 : 0) : (x.i >> y.i));
          break;
      }
    }
  }
  return ORC_OK;
}

// ===========================================================================
// Elementwise: unary operators with scalar parameters (Table 1 "Deep Learning" activations and friends)
// ===========================================================================
// out[i] = f(a[i]; p0, p1, p2); out has a's shape and the result dtype.  The parameters are binary64 values and the
// function is evaluated in binary64 on the input converted to the result dtype, one rounding.
//   leaky_relu(p0 = slope)  : x > 0 ? x : x * slope
//   elu(p0 = alpha)         : x > 0 ? x : alpha * expm1(x)
//   celu(p0 = alpha != 0)   : x > 0 ? x : alpha * expm1(x / alpha)       (alpha = 0 is ORC_ERR_SCALAR)
//   selu                    : scale * (x > 0 ? x : alpha * expm1(x)), scale = 1.0507009873554805, alpha = 1.6732632423543772
//   softplus(p0 = beta, p1 = threshold) : x * beta > threshold ? x : log1p(exp(x * beta)) / beta
//   hardshrink(p0 = lambda) : -lambda <= x <= lambda ? 0 : x                (a NaN stays)
//   softshrink(p0 = lambda >= 0) : x > lambda ? x - lambda : x < -lambda ? x + lambda : x * 0   (keeps -0.0 and NaN;
//                             a negative lambda is ORC_ERR_SCALAR)
//     - these seven take floating dtypes only -
//   threshold(p0 = threshold, p1 = value) : x <= threshold ? value : x; floats and int32 / int64 (the two parameters are
//                             truncated to the integer dtype first); a NaN x stays
//   logit(p0 = eps, p1 != 0: eps given) : log(z / (1 - z)), z = x clamped to [eps, 1 - eps] when eps is given (x < eps ?
//                             eps : x > 1 - eps ? 1 - eps : x); bool / integer input computes in fp32
//   nan_to_num(p0 = nan, p1 = posinf, p2 = neginf) : replaces NaN, +inf, -inf by the parameters rounded to the dtype;
//                             integers and bools are returned as they are
//   round_decimals(p0 = d, an integer) : d > 0: rint(x * 10^d) / 10^d; d < 0: rint(x / 10^-d) * 10^-d; d = 0: rint(x);
//                             halves to even.  The operator is defined by this arithmetic in binary32 (10^|d| rounded
//                             to binary32, each product and quotient rounded to binary32), so it is evaluated that
//                             way here; floating dtypes only
//   gelu_tanh               : x / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3), which is the tanh form
//                             x (1 + tanh u) / 2 written without the cancellation at negative u; floating dtypes only
int orc_unary_param_result_dtype(int op, int in_dtype) {
  if (!valid_dtype(in_dtype)) return ORC_ERR_DTYPE;
  switch (op) {
    case ORC_LEAKY_RELU: case ORC_ELU: case ORC_CELU: case ORC_SELU: case ORC_SOFTPLUS: case ORC_HARDSHRINK: case ORC_SOFTSHRINK:
    case ORC_ROUND_DECIMALS: case ORC_GELU_TANH:
      return is_float(in_dtype) ? in_dtype : ORC_ERR_DTYPE;
    case ORC_THRESHOLD: return in_dtype == ORC_BOOL ? ORC_ERR_DTYPE : in_dtype;
    case ORC_LOGIT: return is_float(in_dtype) ? in_dtype : ORC_F32;
    case ORC_NAN_TO_NUM: return in_dtype;
  }
  return ORC_ERR_SCALAR;
}

int orc_unary_param(int op, const orc_tensor* out, const orc_tensor* a, double p0, double p1, double p2) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(a))) return rc;
  const int rd = orc_unary_param_result_dtype(op, a->dtype);
  if (rd < 0) return rd;
  if (out->dtype != rd) return ORC_ERR_DTYPE;
  if (!same_shape(out, a->ndim, a->sizes)) return ORC_ERR_SHAPE;
  if (op == ORC_CELU && p0 == 0.0) return ORC_ERR_SCALAR;
  if (op == ORC_SOFTSHRINK && !(p0 >= 0.0)) return ORC_ERR_SCALAR;
  if (op == ORC_ROUND_DECIMALS && (p0 != std::trunc(p0) || std::fabs(p0) > 38.0)) return ORC_ERR_SCALAR;
  const float ten_pow = (float)std::pow(10.0, std::fabs(p0));       // round_decimals: 10^|d| in binary32
  const int64_t n = numel(out);
  const int nd = a->ndim;
  const double selu_scale = 1.0507009873554804934193349852946, selu_alpha = 1.6732632423543772848170429916717;
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, out->sizes, idx);
    const int64_t oo = offset_of(out, idx), ao = offset_of(a, idx);
    if (!is_float(rd)) {                                // threshold / nan_to_num of an integer or bool tensor
      const int64_t v = load_int(a, ao);
      if (op == ORC_THRESHOLD) {
        const int64_t th = rd == ORC_I32 ? (int64_t)(int32_t)p0 : (int64_t)p0, val = rd == ORC_I32 ? (int64_t)(int32_t)p1 : (int64_t)p1;
        put_int(out, oo, rd, v <= th ? val : v);
      } else {
        put_int(out, oo, rd, v);
      }
      continue;
    }
    const double x = (double)load_as(a, ao, rd).f;
    double y = 0.0;
    switch (op) {
      case ORC_LEAKY_RELU: y = x > 0.0 ? x : x * p0; break;
      case ORC_ELU: y = x > 0.0 ? x : p0 * std::expm1(x); break;
      case ORC_CELU: y = x > 0.0 ? x : p0 * std::expm1(x / p0); break;
      case ORC_SELU: y = selu_scale * (x > 0.0 ? x : selu_alpha * std::expm1(x)); break;
      case ORC_SOFTPLUS: y = x * p0 > p1 ? x : std::log1p(std::exp(x * p0)) / p0; break;
      case ORC_THRESHOLD: y = x <= p0 ? (double)round_to_float_dtype(p1, rd) : x; break;
      case ORC_HARDSHRINK: y = (x >= -p0 && x <= p0) ? 0.0 : x; break;
      case ORC_SOFTSHRINK: y = x > p0 ? x - p0 : (x < -p0 ? x + p0 : x * 0.0); break;
      case ORC_LOGIT: {
        double z = x;
        if (p1 != 0.0) z = z < p0 ? p0 : (z > 1.0 - p0 ? 1.0 - p0 : z);
        y = std::log(z / (1.0 - z));
        break;
      }
      case ORC_NAN_TO_NUM: y = std::isnan(x) ? p0 : (std::isinf(x) ? (x > 0.0 ? p1 : p2) : x); break;
      case ORC_ROUND_DECIMALS: {
        const float xf = (float)x;
        if (p0 == 0.0) y = std::nearbyint(xf);
        else if (p0 > 0.0) { const float t = xf * ten_pow; y = std::nearbyint(t) / ten_pow; y = (double)(float)y; }
        else { const float t = xf / ten_pow; y = (double)(float)(std::nearbyint(t) * ten_pow); }
        break;
      }
      case ORC_GELU_TANH: {
        const double u = 0.79788456080286535588 * (x + 0.044715 * x * x * x);
        y = x / (1.0 + std::exp(-2.0 * u));
        break;
      }
    }
    put_flt(out, oo, rd, y);
  }
  return ORC_OK;
}

// ===========================================================================
// Elementwise: ternary (addcmul, addcdiv, lerp) with broadcasting and type promotion
// ===========================================================================
//   addcmul : a + value * b * c.  Integer result: wrapping, value truncated to an integer.  bool is a dtype error.
//   addcdiv : a + value * b / c; the promoted dtype must be floating.
//   lerp    : a + w (b - a) for w < 1/2, b - (b - a)(1 - w) otherwise (exact at both ends); w is the tensor c, or the
//             scalar `value` when c is null; every tensor has one floating dtype.
// Operands are converted to the promoted dtype, the expression is evaluated in binary64 and rounded once.
int orc_ternary_result_dtype(int op, const orc_tensor* a, const orc_tensor* b, const orc_tensor* c) {
  if (op < ORC_ADDCMUL || op > ORC_LERP) return ORC_ERR_SCALAR;
  if (!a || !b || (op != ORC_LERP && !c)) return ORC_ERR_NULL;
  if (op == ORC_LERP) {
    if (!is_float(a->dtype) || b->dtype != a->dtype || (c && c->dtype != a->dtype)) return ORC_ERR_DTYPE;
    return a->dtype;
  }
  const orc_tensor* ops[3] = {a, b, c};
  const int rd = result_type(ops, 3);
  if (rd == ORC_BOOL) return ORC_ERR_DTYPE;
  if (op == ORC_ADDCDIV && !is_float(rd)) return ORC_ERR_DTYPE;
  return rd;
}

int orc_ternary(int op, const orc_tensor* out, const orc_tensor* a, const orc_tensor* b, const orc_tensor* c, double value_f,
                int64_t value_i, int value_is_int) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(a)) || (rc = check_tensor(b))) return rc;
  if (c && (rc = check_tensor(c))) return rc;
  const int rd = orc_ternary_result_dtype(op, a, b, c);
  if (rd < 0) return rd;
  if (out->dtype != rd) return ORC_ERR_DTYPE;
  const orc_tensor* ops[3] = {a, b, c};
  int nd;
  int64_t sizes[ORC_MAX_DIMS];
  if ((rc = broadcast_shapes(ops, c ? 3 : 2, &nd, sizes))) return rc;
  if (!same_shape(out, nd, sizes)) return ORC_ERR_SHAPE;
  const double value = value_is_int ? (double)value_i : value_f;
  const int64_t ivalue = value_is_int ? value_i : (int64_t)value_f;      // integer result: truncated
  int64_t n = 1;
  for (int d = 0; d < nd; ++d) n *= sizes[d];
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, sizes, idx);
    const int64_t oo = offset_of(out, idx);
    const Val x = load_as(a, bcast_offset(a, nd, idx), rd), y = load_as(b, bcast_offset(b, nd, idx), rd);
    Val z{0, 0.0f};
    if (c) z = load_as(c, bcast_offset(c, nd, idx), rd);
    if (!is_float(rd)) {
      put_int(out, oo, rd, (int64_t)((uint64_t)x.i + (uint64_t)ivalue * (uint64_t)y.i * (uint64_t)z.i));
      continue;
    }
    const double xd = x.f, yd = y.f, zd = c ? (double)z.f : value;
    double r;
    if (op == ORC_ADDCMUL) r = xd + value * yd * zd;
    else if (op == ORC_ADDCDIV) r = xd + value * yd / zd;
    else r = zd < 0.5 ? xd + zd * (yd - xd) : yd - (yd - xd) * (1.0 - zd);
    put_flt(out, oo, rd, r);
  }
  return ORC_OK;
}

// ===========================================================================
// Shape manipulation with data movement (Table 1 "Shape Manipulation"): copy with conversion, flip, roll, tril / triu
// ===========================================================================
// One element converted to out's dtype and stored.  Between floating dtypes: the value, rounded once.  Integer or
// bool to floating: through binary32, nearest-even.  Floating to integer: truncated toward zero (values outside the
// target range, and NaN, are outside the contract).  Anything to bool: value != 0.  int64 to int32 wraps.  The same
// dtype on both sides copies the bits.
static void convert_element(const orc_tensor* out, int64_t oo, const orc_tensor* x, int64_t xo) {
  if (out->dtype == x->dtype) {
    std::memcpy(mptr(out, oo), cptr(x, xo), esize(x->dtype));
  } else if (is_float(x->dtype)) {
    const double v = load_flt(x, xo);
    if (is_float(out->dtype)) store_flt(out, oo, v);
    else if (out->dtype == ORC_BOOL) store_int(out, oo, v != 0.0);
    else store_int(out, oo, (int64_t)v);
  } else {
    const int64_t v = load_int(x, xo);
    if (is_float(out->dtype)) store_flt(out, oo, (double)(float)v);
    else store_int(out, oo, v);
  }
}

// out = x broadcast to out's shape, converted to out's dtype (clone, contiguous, to, expand made real, copy_)
int orc_copy(const orc_tensor* out, const orc_tensor* x) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  const orc_tensor* ops[2] = {out, x};
  int nd;
  int64_t sizes[ORC_MAX_DIMS];
  if ((rc = broadcast_shapes(ops, 2, &nd, sizes))) return rc;
  if (!same_shape(out, nd, sizes)) return ORC_ERR_SHAPE;          // x may be broadcast, out may not
  const int64_t n = numel(out);
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, sizes, idx);
    convert_element(out, offset_of(out, idx), x, bcast_offset(x, nd, idx));
  }
  return ORC_OK;
}

// out[i] = x[j]: along every dim listed in `dims`, j = size - 1 - i (flip, how = 0), or j = (i - shift) mod size
// (roll, how = 1: the element at j moves to j + shift); other coordinates are equal.  Same shape and dtype; a dim
// listed twice is ORC_ERR_DIM for flip, and shifts add up for roll.
int orc_flip_roll(int how, const orc_tensor* out, const orc_tensor* x, const int64_t* dims, const int64_t* shifts, int32_t n) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  if (out->dtype != x->dtype) return ORC_ERR_DTYPE;
  if (!same_shape(out, x->ndim, x->sizes)) return ORC_ERR_SHAPE;
  const int nd = x->ndim;
  bool flip[ORC_MAX_DIMS] = {false};
  int64_t shift[ORC_MAX_DIMS] = {0};
  for (int i = 0; i < n; ++i) {
    int64_t d = dims[i];
    const int lim = nd == 0 ? 1 : nd;
    if (d < -lim || d >= lim) return ORC_ERR_DIM;
    if (d < 0) d += lim;
    if (nd == 0) continue;                              // a 0-dim tensor has nothing to move
    if (how == 0) {
      if (flip[d]) return ORC_ERR_DIM;
      flip[d] = true;
    } else if (x->sizes[d] > 0) {
      shift[d] = ((shift[d] + shifts[i]) % x->sizes[d] + x->sizes[d]) % x->sizes[d];
    }
  }
  const int64_t total = numel(out);
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < total; ++lin) {
    int64_t idx[ORC_MAX_DIMS], src[ORC_MAX_DIMS];
    unravel(lin, nd, out->sizes, idx);
    for (int d = 0; d < nd; ++d)
      src[d] = flip[d] ? x->sizes[d] - 1 - idx[d] : ((idx[d] - shift[d]) % x->sizes[d] + x->sizes[d]) % x->sizes[d];
    std::memcpy(mptr(out, offset_of(out, idx)), cptr(x, offset_of(x, src)), esize(x->dtype));
  }
  return ORC_OK;
}

// tril (upper = 0): out[..., i, j] = x[..., i, j] where j - i <= diagonal, else 0; triu (upper != 0): where
// j - i >= diagonal.  At least two dims; same shape and dtype.
int orc_tri(const orc_tensor* out, const orc_tensor* x, int64_t diagonal, int upper) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  if (out->dtype != x->dtype) return ORC_ERR_DTYPE;
  if (x->ndim < 2) return ORC_ERR_NDIM;
  if (!same_shape(out, x->ndim, x->sizes)) return ORC_ERR_SHAPE;
  const int nd = x->ndim;
  const int64_t total = numel(out);
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < total; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, out->sizes, idx);
    const int64_t off = idx[nd - 1] - idx[nd - 2];
    const bool keep = upper ? off >= diagonal : off <= diagonal;
    char* dst = mptr(out, offset_of(out, idx));
    if (keep) std::memcpy(dst, cptr(x, offset_of(x, idx)), esize(x->dtype));
    else std::memset(dst, 0, esize(x->dtype));
  }
  return ORC_OK;
}

// where(cond, x, y): cond must be bool; result dtype = promotion of x and y;
// all three broadcast together.  The selected element is converted to the
// result dtype; when no conversion is needed its bits are copied unchanged.
int orc_where(const orc_tensor* out, const orc_tensor* cond, const orc_tensor* x, const orc_tensor* y) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(cond)) || (rc = check_tensor(x)) || (rc = check_tensor(y)))
    return rc;
  if (cond->dtype != ORC_BOOL) return ORC_ERR_DTYPE;
  int rd = orc_where_result_dtype(x, y);
  if (out->dtype != rd) return ORC_ERR_DTYPE;
  const orc_tensor* ops[3] = {cond, x, y};
  int nd;
  int64_t sizes[ORC_MAX_DIMS];
  if ((rc = broadcast_shapes(ops, 3, &nd, sizes))) return rc;
  if (!same_shape(out, nd, sizes)) return ORC_ERR_SHAPE;
  const int64_t n = numel(out);
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, sizes, idx);
    int64_t oo = offset_of(out, idx);
    bool c = load_int(cond, bcast_offset(cond, nd, idx)) != 0;
    const orc_tensor* s = c ? x : y;
    int64_t so = bcast_offset(s, nd, idx);
    if (s->dtype == rd) {
      std::memcpy(mptr(out, oo), cptr(s, so), esize(rd));
    } else {
      Val v = load_as(s, so, rd);
      if (is_float(rd)) store_flt(out, oo, (double)v.f);
      else store_int(out, oo, v.i);
    }
  }
  return ORC_OK;
}

// masked_fill(self, mask, value): out = mask ? value : self.  mask is bool and
// broadcasts with self; `value` is cast to self's dtype (a floating value
// truncates toward zero into an integer dtype; into bool it is value != 0).
int orc_masked_fill(const orc_tensor* out, const orc_tensor* self, const orc_tensor* mask, double value_f,
                    int64_t value_i, int value_is_int) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(self)) || (rc = check_tensor(mask))) return rc;
  if (mask->dtype != ORC_BOOL) return ORC_ERR_DTYPE;
  if (out->dtype != self->dtype) return ORC_ERR_DTYPE;
  const orc_tensor* ops[2] = {self, mask};
  int nd;
  int64_t sizes[ORC_MAX_DIMS];
  if ((rc = broadcast_shapes(ops, 2, &nd, sizes))) return rc;
  if (!same_shape(out, nd, sizes)) return ORC_ERR_SHAPE;
  const int dt = self->dtype;
  // the fill value in self's dtype, encoded once
  char fill[8] = {0};
  {
    orc_tensor tmp;
    tmp.data = fill; tmp.dtype = dt; tmp.ndim = 0;
    if (is_float(dt)) store_flt(&tmp, 0, value_is_int ? (double)value_i : value_f);
    else if (dt == ORC_BOOL) store_int(&tmp, 0, value_is_int ? (value_i != 0) : (value_f != 0.0));
    else store_int(&tmp, 0, value_is_int ? value_i : (int64_t)std::trunc(value_f));
  }
  const int64_t n = numel(out);
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, sizes, idx);
    int64_t oo = offset_of(out, idx);
    bool m = load_int(mask, bcast_offset(mask, nd, idx)) != 0;
    if (m) std::memcpy(mptr(out, oo), fill, esize(dt));
    else std::memcpy(mptr(out, oo), cptr(self, bcast_offset(self, nd, idx)), esize(dt));
  }
  return ORC_OK;
}

// clamp(x, lo, hi) with scalar bounds, either of which may be absent (not both): min(max(x, lo), hi), so a lower
// bound above the upper bound gives the upper bound everywhere.  Result dtype: x's, except that an integer x with
// a floating bound gives fp32; bool x is a dtype error.  x and the bounds are converted to the result dtype first
// (an integer bound that does not fit an integer result dtype is a scalar error); a NaN in x stays, a NaN bound
// makes every output NaN.
int orc_clamp_result_dtype(int x_dtype, int has_lo, int lo_is_int, int has_hi, int hi_is_int) {
  if (!valid_dtype(x_dtype) || x_dtype == ORC_BOOL) return ORC_ERR_DTYPE;
  if (!has_lo && !has_hi) return ORC_ERR_SCALAR;
  if (is_float(x_dtype)) return x_dtype;
  return ((has_lo && !lo_is_int) || (has_hi && !hi_is_int)) ? ORC_F32 : x_dtype;
}
int orc_clamp(const orc_tensor* out, const orc_tensor* x, int has_lo, double lo_f, int64_t lo_i, int lo_is_int,
              int has_hi, double hi_f, int64_t hi_i, int hi_is_int) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  int rd = orc_clamp_result_dtype(x->dtype, has_lo, lo_is_int, has_hi, hi_is_int);
  if (rd < 0) return rd;
  if (!can_cast(rd, out->dtype)) return ORC_ERR_DTYPE;
  if (!same_shape(out, x->ndim, x->sizes)) return ORC_ERR_SHAPE;
  float lof = 0.0f, hif = 0.0f;
  if (is_float(rd)) {
    lof = round_to_float_dtype(lo_is_int ? (double)lo_i : lo_f, rd);
    hif = round_to_float_dtype(hi_is_int ? (double)hi_i : hi_f, rd);
  } else if (rd == ORC_I32) {
    if ((has_lo && (lo_i < INT32_MIN || lo_i > INT32_MAX)) || (has_hi && (hi_i < INT32_MIN || hi_i > INT32_MAX)))
      return ORC_ERR_SCALAR;
  }
  const bool nan_bound = is_float(rd) && ((has_lo && std::isnan(lof)) || (has_hi && std::isnan(hif)));
  const int64_t n = numel(out);
  const int nd = x->ndim;
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, out->sizes, idx);
    int64_t oo = offset_of(out, idx);
    Val v = load_as(x, offset_of(x, idx), rd);
    if (is_float(rd)) {
      float r = v.f;
      if (nan_bound) r = std::numeric_limits<float>::quiet_NaN();
      else if (!std::isnan(r)) {
        if (has_lo && r < lof) r = lof;
        if (has_hi && r > hif) r = hif;
      }
      put_flt(out, oo, rd, (double)r);
    } else {
      int64_t r = v.i;
      if (has_lo && r < lo_i) r = lo_i;
      if (has_hi && r > hi_i) r = hi_i;
      put_int(out, oo, rd, r);
    }
  }
  return ORC_OK;
}

// ===========================================================================
// Reductions
// ===========================================================================
// Normalise a dim list: wrap negatives, reject out-of-range and duplicates.
// An empty list means all dims.  A 0-dim tensor accepts dim 0 / -1.
// logsumexp operand: a floating element as it is, a bool / integer element converted to fp32 (nearest-even)
static inline double lse_value(const orc_tensor* x, int64_t off) {
  return is_float(x->dtype) ? load_flt(x, off) : (double)(float)load_int(x, off);
}

static int normalise_dims(int nd, const int64_t* dims, int ndims, bool* reduced) {
  for (int d = 0; d < ORC_MAX_DIMS; ++d) reduced[d] = false;
  if (ndims == 0 || dims == nullptr) {
    for (int d = 0; d < nd; ++d) reduced[d] = true;
    return ORC_OK;
  }
  int lim = nd == 0 ? 1 : nd;
  bool seen[ORC_MAX_DIMS] = {false};
  for (int i = 0; i < ndims; ++i) {
    int64_t d = dims[i];
    if (d < -lim || d >= lim) return ORC_ERR_DIM;
    if (d < 0) d += lim;
    if (seen[d]) return ORC_ERR_DIM;
    seen[d] = true;
    if (nd > 0) reduced[d] = true;
  }
  return ORC_OK;
}

int orc_reduce_result_dtype(int op, int in_dtype) {
  if (!valid_dtype(in_dtype)) return ORC_ERR_DTYPE;
  switch (op) {
    case ORC_SUM: case ORC_PROD: return is_float(in_dtype) ? in_dtype : ORC_I64;
    case ORC_MEAN: case ORC_VAR: case ORC_STD: return is_float(in_dtype) ? in_dtype : ORC_ERR_DTYPE;
    case ORC_LOGSUMEXP: return is_float(in_dtype) ? in_dtype : ORC_F32;    // bool / integer input is converted to fp32
    case ORC_AMAX: case ORC_AMIN: return in_dtype;
    case ORC_ARGMAX: case ORC_ARGMIN: return in_dtype == ORC_BOOL ? (int)ORC_ERR_DTYPE : (int)ORC_I64;
    case ORC_ANY: case ORC_ALL: return ORC_BOOL;
    case ORC_NANSUM: return is_float(in_dtype) ? in_dtype : ORC_I64;
    case ORC_NANMEAN: case ORC_NORM: return is_float(in_dtype) ? in_dtype : ORC_ERR_DTYPE;
    case ORC_COUNT_NONZERO: return ORC_I64;
  }
  return ORC_ERR_DTYPE;
}

int orc_infer_reduce(int op, const orc_tensor* x, const int64_t* dims, int32_t ndims, int keepdim, int32_t* dtype,
                     int32_t* ndim, int64_t* sizes) {
  if (!x) return ORC_ERR_NULL;
  if (x->ndim < 0 || x->ndim > ORC_MAX_DIMS) return ORC_ERR_NDIM;
  int rd = orc_reduce_result_dtype(op, x->dtype);
  if (rd < 0) return rd;
  bool all = (ndims == 0 || dims == nullptr);
  if ((op == ORC_PROD || op == ORC_ARGMAX || op == ORC_ARGMIN) && ndims > 1) return ORC_ERR_DIM;  // single dim or all
  bool red[ORC_MAX_DIMS];
  int rc = normalise_dims(x->ndim, dims, ndims, red);
  if (rc) return rc;
  (void)all;
  int nd = 0;
  for (int d = 0; d < x->ndim; ++d) {
    if (red[d]) { if (keepdim) sizes[nd++] = 1; }
    else sizes[nd++] = x->sizes[d];
  }
  if (dtype) *dtype = rd;
  if (ndim) *ndim = nd;
  return ORC_OK;
}

// Reduce x over `dims` (all dims when ndims == 0).
//   sum   : integers/bool accumulate exactly in int64 (wrapping); floats
//           accumulate sequentially in binary64, one rounding.
//   mean  : that sum divided by the count (NaN for an empty extent).
//   prod  : like sum with multiplication; empty product = 1.
//   amax  : maximum, NaN if any element is NaN; empty reduced extent: error.
//   argmax: index (along the one dim, or flat row-major over the logical
//           shape) of the maximum; ties -> lowest index; NaN ranks above
//           everything and the first NaN wins.  int64 result.
//   var   : two passes in binary64: mean, then sum of squared deviations,
//           divided by max(0, n - correction).
//   std   : the square root of that variance.
//   amin / argmin : amax / argmax with the order reversed (NaN still wins,
//           ties still go to the lowest index).
//   any / all : whether some / every element is non-zero (NaN is non-zero);
//           any input dtype, bool result; empty extent: any = false, all = true.
//   logsumexp : max + log(sum exp(x - max)) in binary64; an infinite maximum is
//           the result (-inf for an empty or all -inf slice), NaN is sticky.
//   nansum / nanmean : sum and mean of the elements that are not NaN (the mean
//           divides by their count: NaN when there is none); nansum of an
//           integer tensor is its sum; nanmean takes floats only.
//   count_nonzero : the number of elements that are not zero (a NaN is not
//           zero, -0.0 is); any dtype, int64 result.
//   norm  : the vector p-norm with p = `correction`; floats only.  p = 0: the
//           count of non-zero elements; p = +inf / -inf: the largest / smallest
//           |x| (NaN if any NaN; empty extent: error); otherwise
//           (sum |x|^p)^(1/p) in binary64 - p = 1 and p = 2 written as |x| and
//           x*x with a square root - so nothing overflows that the result does
//           not; a negative p over an empty extent is an error as well.
// A floating `out` dtype wider than x's (fp32 out for a half x) is allowed for
// sum / mean / prod / var: the single rounding then goes to that dtype.
int orc_reduce(int op, const orc_tensor* out, const orc_tensor* x, const int64_t* dims, int32_t ndims, int keepdim,
               double correction) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  int32_t rd, ond;
  int64_t osz[ORC_MAX_DIMS];
  if ((rc = orc_infer_reduce(op, x, dims, ndims, keepdim, &rd, &ond, osz))) return rc;
  bool widen_ok = is_float(rd) && out->dtype == ORC_F32 && op != ORC_AMAX && op != ORC_AMIN;
  if (out->dtype != rd && !widen_ok) return ORC_ERR_DTYPE;
  if (!same_shape(out, ond, osz)) return ORC_ERR_SHAPE;
  bool red[ORC_MAX_DIMS];
  normalise_dims(x->ndim, dims, ndims, red);
  const int nd = x->ndim;
  // kept and reduced dim lists in logical order
  int kd[ORC_MAX_DIMS], rdm[ORC_MAX_DIMS], nk = 0, nr = 0;
  int64_t ksz[ORC_MAX_DIMS], rsz[ORC_MAX_DIMS];
  for (int d = 0; d < nd; ++d) {
    if (red[d]) { rdm[nr] = d; rsz[nr++] = x->sizes[d]; }
    else { kd[nk] = d; ksz[nk++] = x->sizes[d]; }
  }
  int64_t nout = 1, nred = 1;
  for (int i = 0; i < nk; ++i) nout *= ksz[i];
  for (int i = 0; i < nr; ++i) nred *= rsz[i];
  if (nout == 0) return ORC_OK;
  if ((op == ORC_AMAX || op == ORC_ARGMAX || op == ORC_AMIN || op == ORC_ARGMIN) && nred == 0)
    return ORC_ERR_EMPTY_REDUCTION;
  const double ord = correction;                       // norm: the exponent p
  if (op == ORC_NORM && std::isnan(ord)) return ORC_ERR_SCALAR;
  if (op == ORC_NORM && nred == 0 && (std::isinf(ord) || ord < 0.0)) return ORC_ERR_EMPTY_REDUCTION;
  const bool flt = is_float(x->dtype);
  const bool single_dim = (nr == 1);

#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < nout; ++o) {
    int64_t kidx[ORC_MAX_DIMS], ridx[ORC_MAX_DIMS], xi[ORC_MAX_DIMS], oi[ORC_MAX_DIMS];
    unravel(o, nk, ksz, kidx);
    for (int i = 0; i < nk; ++i) xi[kd[i]] = kidx[i];
    // output multi-index
    {
      int p = 0, k = 0;
      for (int d = 0; d < nd; ++d) {
        if (red[d]) { if (keepdim) oi[p++] = 0; }
        else oi[p++] = kidx[k++];
      }
    }
    const int64_t oo = offset_of(out, oi);

    double accd = (op == ORC_PROD) ? 1.0 : 0.0;
    uint64_t acci = (op == ORC_PROD) ? 1u : 0u;
    bool have = false, isnan_best = false;
    double bestd = 0.0;
    int64_t besti = 0, bestpos = 0;
    double mean = 0.0;
    bool any_true = false, all_true = true;            // any / all: an element counts as true when it is not zero (NaN is)
    double lse_max = -std::numeric_limits<double>::infinity();
    bool lse_nan = false;
    int64_t count = 0;                                 // nanmean: elements that are not NaN; count_nonzero, norm 0: not zero
    bool norm_nan = false;
    if (op == ORC_LOGSUMEXP) {                         // first pass: the maximum (NaN is sticky)
      for (int64_t r = 0; r < nred; ++r) {
        unravel(r, nr, rsz, ridx);
        for (int i = 0; i < nr; ++i) xi[rdm[i]] = ridx[i];
        double v = lse_value(x, offset_of(x, xi));
        if (std::isnan(v)) lse_nan = true;
        else if (v > lse_max) lse_max = v;
      }
    }
    if (op == ORC_VAR || op == ORC_STD) {
      double s = 0.0;
      for (int64_t r = 0; r < nred; ++r) {
        unravel(r, nr, rsz, ridx);
        for (int i = 0; i < nr; ++i) xi[rdm[i]] = ridx[i];
        s += load_flt(x, offset_of(x, xi));
      }
      mean = s / (double)nred;
    }
    for (int64_t r = 0; r < nred; ++r) {
      unravel(r, nr, rsz, ridx);
      for (int i = 0; i < nr; ++i) xi[rdm[i]] = ridx[i];
      const int64_t xo = offset_of(x, xi);
      const int64_t pos = single_dim ? ridx[0] : r;
      switch (op) {
        case ORC_SUM: case ORC_MEAN:
          if (flt) accd += load_flt(x, xo); else acci += (uint64_t)load_int(x, xo);
          break;
        case ORC_PROD:
          if (flt) accd *= load_flt(x, xo); else acci *= (uint64_t)load_int(x, xo);
          break;
        case ORC_VAR: case ORC_STD: {
          double dlt = load_flt(x, xo) - mean;
          accd += dlt * dlt;
          break;
        }
        case ORC_NANSUM: case ORC_NANMEAN:
          if (flt) {
            const double v = load_flt(x, xo);
            if (!std::isnan(v)) { accd += v; ++count; }
          } else {
            acci += (uint64_t)load_int(x, xo);
          }
          break;
        case ORC_COUNT_NONZERO:
          count += flt ? (load_flt(x, xo) != 0.0) : (load_int(x, xo) != 0);
          break;
        case ORC_NORM: {
          const double v = std::fabs(load_flt(x, xo));
          if (ord == 0.0) count += (v != 0.0);                           // NaN != 0 is true
          else if (std::isinf(ord)) {
            if (std::isnan(v)) norm_nan = true;
            else if (!have || (ord > 0.0 ? v > bestd : v < bestd)) { bestd = v; have = true; }
          }
          else if (ord == 1.0) accd += v;
          else if (ord == 2.0) accd += v * v;
          else accd += std::pow(v, ord);
          break;
        }
        case ORC_ANY: case ORC_ALL: {
          bool t = flt ? (load_flt(x, xo) != 0.0) : (load_int(x, xo) != 0);     // NaN != 0 is true
          any_true = any_true || t;
          all_true = all_true && t;
          break;
        }
        case ORC_LOGSUMEXP:                            // second pass: sum of exp(x - max); skipped when max is infinite
          if (std::isfinite(lse_max)) accd += std::exp(lse_value(x, xo) - lse_max);
          break;
        case ORC_AMIN: case ORC_ARGMIN:
          if (flt) {
            double v = load_flt(x, xo);
            if (!have) { bestd = v; bestpos = pos; have = true; isnan_best = std::isnan(v); }
            else if (!isnan_best && (std::isnan(v) || v < bestd)) { bestd = v; bestpos = pos; isnan_best = std::isnan(v); }
          } else {
            int64_t v = load_int(x, xo);
            if (!have || v < besti) { besti = v; bestpos = pos; have = true; }
          }
          break;
        case ORC_AMAX: case ORC_ARGMAX:
          if (flt) {
            double v = load_flt(x, xo);
            if (!have) { bestd = v; bestpos = pos; have = true; isnan_best = std::isnan(v); }
            else if (!isnan_best && (std::isnan(v) || v > bestd)) { bestd = v; bestpos = pos; isnan_best = std::isnan(v); }
          } else {
            int64_t v = load_int(x, xo);
            if (!have || v > besti) { besti = v; bestpos = pos; have = true; }
          }
          break;
      }
    }
    switch (op) {
      case ORC_SUM: case ORC_PROD:
        if (flt) store_flt(out, oo, accd); else store_int(out, oo, (int64_t)acci);
        break;
      case ORC_MEAN:
        store_flt(out, oo, nred ? accd / (double)nred : kNaN);
        break;
      case ORC_VAR: {
        double div = (double)nred - correction;
        if (div < 0.0) div = 0.0;
        store_flt(out, oo, nred ? accd / div : kNaN);
        break;
      }
      case ORC_STD: {
        double div = (double)nred - correction;
        if (div < 0.0) div = 0.0;
        store_flt(out, oo, nred ? std::sqrt(accd / div) : kNaN);
        break;
      }
      case ORC_NANSUM:
        if (flt) store_flt(out, oo, accd); else store_int(out, oo, (int64_t)acci);
        break;
      case ORC_NANMEAN: store_flt(out, oo, count ? accd / (double)count : kNaN); break;
      case ORC_COUNT_NONZERO: store_int(out, oo, count); break;
      case ORC_NORM:
        if (ord == 0.0) store_flt(out, oo, (double)count);
        else if (std::isinf(ord)) store_flt(out, oo, norm_nan ? kNaN : bestd);
        else if (ord == 1.0) store_flt(out, oo, accd);
        else if (ord == 2.0) store_flt(out, oo, std::sqrt(accd));
        else store_flt(out, oo, std::pow(accd, 1.0 / ord));
        break;
      case ORC_ANY: store_int(out, oo, any_true); break;
      case ORC_ALL: store_int(out, oo, all_true); break;
      case ORC_LOGSUMEXP:
        // log sum exp(x) = max + log sum exp(x - max); an infinite maximum is the result itself
        // (-inf for an empty or all -inf slice, +inf when +inf is present), NaN is sticky
        if (lse_nan) store_flt(out, oo, kNaN);
        else if (!std::isfinite(lse_max)) store_flt(out, oo, lse_max);
        else store_flt(out, oo, lse_max + std::log(accd));
        break;
      case ORC_AMAX: case ORC_AMIN:
        if (flt) store_flt(out, oo, bestd); else store_int(out, oo, besti);
        break;
      case ORC_ARGMAX: case ORC_ARGMIN:
        store_int(out, oo, bestpos);
        break;
    }
  }
  return ORC_OK;
}

// ===========================================================================
// softmax / log_softmax along one dim
// ===========================================================================
// m = max over the slice; softmax = exp(x-m) / sum exp(x-m);
// log_softmax = (x-m) - log sum exp(x-m).  binary64 throughout, one rounding.
// IEEE arithmetic gives the special cases: a -inf entry -> 0 / -inf; a slice
// that is all -inf, or contains +inf or NaN -> all NaN.  `out` may be fp32 for
// a half input (the dtype= variant).
int orc_softmax(const orc_tensor* out, const orc_tensor* x, int64_t dim, int is_log) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  if (!is_float(x->dtype)) return ORC_ERR_DTYPE;
  if (out->dtype != x->dtype && out->dtype != ORC_F32) return ORC_ERR_DTYPE;
  if (!same_shape(out, x->ndim, x->sizes)) return ORC_ERR_SHAPE;
  const int nd = x->ndim;
  int lim = nd == 0 ? 1 : nd;
  if (dim < -lim || dim >= lim) return ORC_ERR_DIM;
  if (dim < 0) dim += lim;
  const int64_t L = nd == 0 ? 1 : x->sizes[dim];
  const int64_t xs = nd == 0 ? 0 : x->strides[dim], os = nd == 0 ? 0 : out->strides[dim];
  // the other dims
  int64_t osz[ORC_MAX_DIMS];
  int od[ORC_MAX_DIMS], nod = 0;
  for (int d = 0; d < nd; ++d) if (d != dim) { od[nod] = d; osz[nod++] = x->sizes[d]; }
  int64_t nslices = 1;
  for (int i = 0; i < nod; ++i) nslices *= osz[i];
  if (nslices == 0 || L == 0) return ORC_OK;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < nslices; ++s) {
    int64_t sidx[ORC_MAX_DIMS], xi[ORC_MAX_DIMS] = {0};
    unravel(s, nod, osz, sidx);
    for (int i = 0; i < nod; ++i) xi[od[i]] = sidx[i];
    const int64_t xb = offset_of(x, xi), ob = offset_of(out, xi);
    double m = -kInf;
    bool anynan = false;
    for (int64_t j = 0; j < L; ++j) {
      double v = load_flt(x, xb + j * xs);
      if (std::isnan(v)) anynan = true;
      if (v > m) m = v;
    }
    if (anynan) m = kNaN;
    double sum = 0.0;
    for (int64_t j = 0; j < L; ++j) sum += std::exp(load_flt(x, xb + j * xs) - m);
    const double lsum = std::log(sum);
    for (int64_t j = 0; j < L; ++j) {
      double d = load_flt(x, xb + j * xs) - m;
      store_flt(out, ob + j * os, is_log ? d - lsum : std::exp(d) / sum);
    }
  }
  return ORC_OK;
}

// ===========================================================================
// layer_norm over the last k dims (the listing of Appendix B.3 is the paper's kernel for this operator)
// ===========================================================================
// The last `norm_ndim` dims of x form one row of M elements; for every row
//   mean = sum x / M,  var = sum (x - mean)^2 / M  (biased),
//   y = (x - mean) / sqrt(var + eps) * weight + bias,
// weight and bias optional (null), each with exactly the shape of the normalised dims, floating dtype.  binary64
// throughout, two passes over the row, one rounding to out's dtype (= x's).  Rows of no elements give no output.
int orc_layer_norm(const orc_tensor* out, const orc_tensor* x, int32_t norm_ndim, const orc_tensor* weight,
                   const orc_tensor* bias, double eps) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  if (weight && (rc = check_tensor(weight))) return rc;
  if (bias && (rc = check_tensor(bias))) return rc;
  if (!is_float(x->dtype) || out->dtype != x->dtype) return ORC_ERR_DTYPE;
  if ((weight && !is_float(weight->dtype)) || (bias && !is_float(bias->dtype))) return ORC_ERR_DTYPE;
  if (!same_shape(out, x->ndim, x->sizes)) return ORC_ERR_SHAPE;
  const int nd = x->ndim;
  if (norm_ndim < 1 || norm_ndim > nd) return ORC_ERR_DIM;
  const int lead = nd - norm_ndim;
  if (weight && !same_shape(weight, norm_ndim, x->sizes + lead)) return ORC_ERR_SHAPE;
  if (bias && !same_shape(bias, norm_ndim, x->sizes + lead)) return ORC_ERR_SHAPE;
  int64_t rows = 1, M = 1;
  for (int d = 0; d < lead; ++d) rows *= x->sizes[d];
  for (int d = lead; d < nd; ++d) M *= x->sizes[d];
  if (rows == 0 || M == 0) return ORC_OK;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(r, lead, x->sizes, idx);
    double sum = 0.0;
    for (int64_t j = 0; j < M; ++j) {
      unravel(j, norm_ndim, x->sizes + lead, idx + lead);
      sum += load_flt(x, offset_of(x, idx));
    }
    const double mean = sum / (double)M;
    double sq = 0.0;
    for (int64_t j = 0; j < M; ++j) {
      unravel(j, norm_ndim, x->sizes + lead, idx + lead);
      const double d = load_flt(x, offset_of(x, idx)) - mean;
      sq += d * d;
    }
    const double rstd = 1.0 / std::sqrt(sq / (double)M + eps);
    for (int64_t j = 0; j < M; ++j) {
      unravel(j, norm_ndim, x->sizes + lead, idx + lead);
      double y = (load_flt(x, offset_of(x, idx)) - mean) * rstd;
      if (weight) y *= load_flt(weight, offset_of(weight, idx + lead));
      if (bias) y += load_flt(bias, offset_of(bias, idx + lead));
      store_flt(out, offset_of(out, idx), y);
    }
  }
  return ORC_OK;
}

// ===========================================================================
// binary_cross_entropy (the listing of Appendix B.1 is the paper's kernel for this operator)
// ===========================================================================
// loss = -weight * (t * max(ln x, -100) + (1 - t) * max(ln(1 - x), -100)); the clamp at -100 keeps x = 0 and
// x = 1 finite; a NaN passes through.  x and t have the same shape and floating dtype; weight is optional (null)
// and broadcasts to that shape.  x is meant to lie in [0, 1]; this is not checked, the formula is applied as it
// stands.  reduction: 0 none (out has x's shape), 1 mean, 2 sum (out is 0-dim; the mean of no elements is NaN,
// the sum 0).  ln(1 - x) is taken as log1p(-x).  binary64 throughout (the sum is one running binary64
// accumulator), one rounding to out's dtype (= x's).
int orc_bce(const orc_tensor* out, const orc_tensor* x, const orc_tensor* t, const orc_tensor* weight, int reduction) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x)) || (rc = check_tensor(t))) return rc;
  if (weight && (rc = check_tensor(weight))) return rc;
  if (!is_float(x->dtype) || t->dtype != x->dtype || out->dtype != x->dtype) return ORC_ERR_DTYPE;
  if (weight && !is_float(weight->dtype)) return ORC_ERR_DTYPE;
  if (reduction < 0 || reduction > 2) return ORC_ERR_SCALAR;
  if (!same_shape(t, x->ndim, x->sizes)) return ORC_ERR_SHAPE;
  if (weight) {
    const orc_tensor* ops[2] = {x, weight};
    int nd;
    int64_t sizes[ORC_MAX_DIMS];
    if ((rc = broadcast_shapes(ops, 2, &nd, sizes))) return rc;
    if (!same_shape(x, nd, sizes)) return ORC_ERR_SHAPE;           // weight may not enlarge the shape
  }
  if (reduction == 0 ? !same_shape(out, x->ndim, x->sizes) : out->ndim != 0) return ORC_ERR_SHAPE;
  const int64_t n = numel(x);
  const int nd = x->ndim;
  auto loss_at = [&](int64_t lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, x->sizes, idx);
    const double xv = load_flt(x, offset_of(x, idx)), tv = load_flt(t, offset_of(t, idx));
    double lx = std::log(xv), l1x = std::log1p(-xv);
    if (lx < -100.0) lx = -100.0;
    if (l1x < -100.0) l1x = -100.0;
    double l = -(tv * lx + (1.0 - tv) * l1x);
    if (weight) l *= load_flt(weight, bcast_offset(weight, nd, idx));
    return l;
  };
  if (reduction == 0) {
#pragma omp parallel for schedule(static)
    for (int64_t lin = 0; lin < n; ++lin) {
      int64_t idx[ORC_MAX_DIMS];
      unravel(lin, nd, x->sizes, idx);
      store_flt(out, offset_of(out, idx), loss_at(lin));
    }
    return ORC_OK;
  }
  double sum = 0.0;
  for (int64_t lin = 0; lin < n; ++lin) sum += loss_at(lin);
  store_flt(out, 0, reduction == 1 ? sum / (double)n : sum);
  return ORC_OK;
}

// ===========================================================================
// regression losses: mse_loss, l1_loss, smooth_l1_loss, huber_loss (Table 1 "Deep Learning"; the same
// elementwise-term-then-reduce shape as the binary_cross_entropy listing of Appendix B.1)
// ===========================================================================
// With d = x - t on the broadcast of the two shapes:
//   kind 0 mse       : d^2
//   kind 1 l1        : |d|
//   kind 2 smooth_l1 : |d| < beta ? d^2 / (2 beta) : |d| - beta / 2   (param = beta >= 0; beta = 0 is l1)
//   kind 3 huber     : |d| <= delta ? d^2 / 2 : delta (|d| - delta / 2)   (param = delta > 0)
// A parameter outside its range is ORC_ERR_SCALAR.  x and t have one floating dtype, which is out's too.
// reduction: 0 none (out has the broadcast shape), 1 mean, 2 sum (out is 0-dim; the mean of no elements is NaN,
// the sum 0).  binary64 throughout (the sum is one running binary64 accumulator), one rounding to out's dtype.
int orc_loss(int kind, const orc_tensor* out, const orc_tensor* x, const orc_tensor* t, int reduction, double param) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x)) || (rc = check_tensor(t))) return rc;
  if (kind < 0 || kind > 3) return ORC_ERR_SCALAR;
  if (!is_float(x->dtype) || t->dtype != x->dtype || out->dtype != x->dtype) return ORC_ERR_DTYPE;
  if (reduction < 0 || reduction > 2) return ORC_ERR_SCALAR;
  if ((kind == 2 && !(param >= 0.0)) || (kind == 3 && !(param > 0.0))) return ORC_ERR_SCALAR;
  const orc_tensor* ops[2] = {x, t};
  int nd;
  int64_t sizes[ORC_MAX_DIMS];
  if ((rc = broadcast_shapes(ops, 2, &nd, sizes))) return rc;
  if (reduction == 0 ? !same_shape(out, nd, sizes) : out->ndim != 0) return ORC_ERR_SHAPE;
  int64_t n = 1;
  for (int d = 0; d < nd; ++d) n *= sizes[d];
  auto loss_at = [&](int64_t lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, sizes, idx);
    const double d = load_flt(x, bcast_offset(x, nd, idx)) - load_flt(t, bcast_offset(t, nd, idx));
    const double ad = std::fabs(d);
    switch (kind) {
      case 0: return d * d;
      case 1: return ad;
      case 2: return ad < param ? d * d / (2.0 * param) : ad - param / 2.0;     // NaN fails the comparison and comes out of the second form
      default: return ad <= param ? d * d / 2.0 : (std::isnan(ad) ? ad : param * (ad - param / 2.0));
    }
  };
  if (reduction == 0) {
#pragma omp parallel for schedule(static)
    for (int64_t lin = 0; lin < n; ++lin) {
      int64_t idx[ORC_MAX_DIMS];
      unravel(lin, nd, sizes, idx);
      store_flt(out, offset_of(out, idx), loss_at(lin));
    }
    return ORC_OK;
  }
  double sum = 0.0;
  for (int64_t lin = 0; lin < n; ++lin) sum += loss_at(lin);
  store_flt(out, 0, reduction == 1 ? sum / (double)n : sum);
  return ORC_OK;
}

// ===========================================================================
// cumsum along one dim (inclusive)
// ===========================================================================
// bool / int32 / int64 input -> int64 output, exact wrapping sums.  Floating
// input: running binary64 accumulator, each prefix rounded independently to
// the output dtype (x's dtype, or fp32 for a half x).
// cumprod and logcumsumexp along one dim (inclusive), with cumsum's shape and dim rules.
//   op 1 cumprod      : dtypes as cumsum (bool / integer input -> int64, wrapping products); floating input: running
//                       binary64 product, each prefix rounded independently.
//   op 2 logcumsumexp : floating input only; out[i] = log(sum_{j <= i} exp(x[j])), carried as the running maximum m and
//                       the sum s of exp(x[j] - m) in binary64 (out[i] = m + log s); an infinite maximum is the result
//                       itself (-inf while nothing but -inf has been seen), a NaN makes every later prefix NaN.
//   op 0 is cumsum.
int orc_scan(int op, const orc_tensor* out, const orc_tensor* x, int64_t dim) {
  if (op < 0 || op > 2) return ORC_ERR_SCALAR;
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  const bool flt = is_float(x->dtype);
  if (op == 2 && !flt) return ORC_ERR_DTYPE;
  if (flt) { if (out->dtype != x->dtype && out->dtype != ORC_F32) return ORC_ERR_DTYPE; }
  else if (out->dtype != ORC_I64) return ORC_ERR_DTYPE;
  if (!same_shape(out, x->ndim, x->sizes)) return ORC_ERR_SHAPE;
  const int nd = x->ndim;
  int lim = nd == 0 ? 1 : nd;
  if (dim < -lim || dim >= lim) return ORC_ERR_DIM;
  if (dim < 0) dim += lim;
  const int64_t L = nd == 0 ? 1 : x->sizes[dim];
  const int64_t xs = nd == 0 ? 0 : x->strides[dim], os = nd == 0 ? 0 : out->strides[dim];
  int64_t osz[ORC_MAX_DIMS];
  int od[ORC_MAX_DIMS], nod = 0;
  for (int d = 0; d < nd; ++d) if (d != dim) { od[nod] = d; osz[nod++] = x->sizes[d]; }
  int64_t nslices = 1;
  for (int i = 0; i < nod; ++i) nslices *= osz[i];
  if (nslices == 0 || L == 0) return ORC_OK;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < nslices; ++s) {
    int64_t sidx[ORC_MAX_DIMS], xi[ORC_MAX_DIMS] = {0};
    unravel(s, nod, osz, sidx);
    for (int i = 0; i < nod; ++i) xi[od[i]] = sidx[i];
    const int64_t xb = offset_of(x, xi), ob = offset_of(out, xi);
    double accd = op == 1 ? 1.0 : 0.0;
    uint64_t acci = op == 1 ? 1u : 0u;
    double m = -kInf, sum = 0.0;                       // logcumsumexp: running maximum and scaled sum
    bool nan = false;
    for (int64_t j = 0; j < L; ++j) {
      if (op == 2) {
        const double v = load_flt(x, xb + j * xs);
        if (std::isnan(v)) nan = true;
        if (!nan) {
          if (v > m) {                                 // rescale the sum to the new maximum (exp(-inf - finite) = 0 for the first element)
            sum = std::isinf(v) ? 0.0 : sum * std::exp(m - v) + 1.0;
            m = v;
          } else if (!std::isinf(v)) {                 // v <= m, finite: m is finite too
            sum += std::exp(v - m);
          }
        }
        store_flt(out, ob + j * os, nan ? kNaN : (std::isinf(m) ? m : m + std::log(sum)));
      } else if (flt) {
        const double v = load_flt(x, xb + j * xs);
        accd = op == 1 ? accd * v : accd + v;
        store_flt(out, ob + j * os, accd);
      } else {
        const uint64_t v = (uint64_t)load_int(x, xb + j * xs);
        acci = op == 1 ? acci * v : acci + v;
        store_int(out, ob + j * os, (int64_t)acci);
      }
    }
  }
  return ORC_OK;
}

int orc_cumsum(const orc_tensor* out, const orc_tensor* x, int64_t dim) { return orc_scan(0, out, x, dim); }

// ===========================================================================
// Indexing
// ===========================================================================
static inline bool index_dtype_ok(int dt) { return dt == ORC_I32 || dt == ORC_I64; }

// gather: out[i0..] = src[i0.. with coordinate `dim` replaced by index[i0..]].
// out has index's shape and src's dtype.  No negative-index wrap-around.
int orc_gather(const orc_tensor* out, const orc_tensor* src, int64_t dim, const orc_tensor* index) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(src)) || (rc = check_tensor(index))) return rc;
  if (!index_dtype_ok(index->dtype)) return ORC_ERR_DTYPE;
  if (out->dtype != src->dtype) return ORC_ERR_DTYPE;
  // ranks must agree, a 0-dim tensor counting as 1-D with one element
  if (std::max<int>(index->ndim, 1) != std::max<int>(src->ndim, 1)) return ORC_ERR_SHAPE;
  const int nd = src->ndim;
  int lim = nd == 0 ? 1 : nd;
  if (dim < -lim || dim >= lim) return ORC_ERR_DIM;
  if (dim < 0) dim += lim;
  for (int d = 0; d < nd; ++d)
    if (d != dim && index->ndim && index->sizes[d] > src->sizes[d]) return ORC_ERR_SHAPE;
  if (!same_shape(out, index->ndim, index->sizes)) return ORC_ERR_SHAPE;
  const int64_t n = numel(out);
  const int64_t extent = nd == 0 ? 1 : src->sizes[dim];
  const int es = esize(src->dtype);
  int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, out->ndim, out->sizes, idx);
    int64_t oo = offset_of(out, idx);
    int64_t k = load_int(index, offset_of(index, idx));
    if (k < 0 || k >= extent) { bad |= 1; continue; }
    if (nd) idx[dim] = k;
    std::memcpy(mptr(out, oo), cptr(src, offset_of(src, idx)), es);    // a 0-dim src has no coordinates: offset 0
  }
  return bad ? ORC_ERR_INDEX : ORC_OK;
}

// index_select: out = src with extent `dim` replaced by len(index); slice j of
// out along dim is slice index[j] of src.  index is 1-D (or 0-dim = length 1).
int orc_index_select(const orc_tensor* out, const orc_tensor* src, int64_t dim, const orc_tensor* index) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(src)) || (rc = check_tensor(index))) return rc;
  if (!index_dtype_ok(index->dtype)) return ORC_ERR_DTYPE;
  if (out->dtype != src->dtype) return ORC_ERR_DTYPE;
  if (index->ndim > 1) return ORC_ERR_SHAPE;
  const int nd = src->ndim;
  int lim = nd == 0 ? 1 : nd;
  if (dim < -lim || dim >= lim) return ORC_ERR_DIM;
  if (dim < 0) dim += lim;
  const int64_t ni = index->ndim == 0 ? 1 : index->sizes[0];
  const int64_t istride = index->ndim == 0 ? 0 : index->strides[0];
  if (nd == 0) {
    if (ni != 1 || out->ndim != 0) return ORC_ERR_SHAPE;
  } else {
    if (out->ndim != nd) return ORC_ERR_SHAPE;
    for (int d = 0; d < nd; ++d)
      if (out->sizes[d] != (d == dim ? ni : src->sizes[d])) return ORC_ERR_SHAPE;
  }
  const int64_t n = numel(out);
  const int64_t extent = nd == 0 ? 1 : src->sizes[dim];
  const int es = esize(src->dtype);
  int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, nd, out->sizes, idx);
    int64_t oo = offset_of(out, idx);
    int64_t j = nd ? idx[dim] : 0;
    int64_t k = load_int(index, j * istride);
    if (k < 0 || k >= extent) { bad |= 1; continue; }
    if (nd) idx[dim] = k;
    std::memcpy(mptr(out, oo), cptr(src, offset_of(src, idx)), es);
  }
  return bad ? ORC_ERR_INDEX : ORC_OK;
}

// scatter_add_ (in place on self): for every position p of index,
//   self[p with coordinate dim = index[p]] += src[p].
// integers / bool: exact, in position order (bool: OR).  Floating dtypes: the
// contributions of each destination element are accumulated in binary64 in
// position order, the initial value of self is added, one rounding.
int orc_scatter_add(const orc_tensor* self, int64_t dim, const orc_tensor* index, const orc_tensor* src) {
  int rc;
  if ((rc = check_tensor(self)) || (rc = check_tensor(index)) || (rc = check_tensor(src))) return rc;
  if (!index_dtype_ok(index->dtype)) return ORC_ERR_DTYPE;
  if (self->dtype != src->dtype) return ORC_ERR_DTYPE;
  if (index->ndim != self->ndim || src->ndim != self->ndim) return ORC_ERR_SHAPE;
  const int nd = self->ndim;
  int lim = nd == 0 ? 1 : nd;
  if (dim < -lim || dim >= lim) return ORC_ERR_DIM;
  if (dim < 0) dim += lim;
  for (int d = 0; d < nd; ++d) {
    if (index->sizes[d] > src->sizes[d]) return ORC_ERR_SHAPE;
    if (d != dim && index->sizes[d] > self->sizes[d]) return ORC_ERR_SHAPE;
  }
  const int64_t n = numel(index);
  if (n == 0) return ORC_OK;
  const int64_t extent = nd == 0 ? 1 : self->sizes[dim];
  // validate all indices first so that nothing is written on error
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, nd, index->sizes, idx);
    int64_t k = load_int(index, offset_of(index, idx));
    if (k < 0 || k >= extent) return ORC_ERR_INDEX;
  }
  const bool flt = is_float(self->dtype);
  const int64_t nself = numel(self);
  std::vector<double> acc;
  std::vector<uint8_t> touched;
  int64_t lstr[ORC_MAX_DIMS];                          // row-major strides of self's logical shape
  if (flt) {
    acc.assign((size_t)nself, 0.0);
    touched.assign((size_t)nself, 0);
    int64_t s = 1;
    for (int d = nd - 1; d >= 0; --d) { lstr[d] = s; s *= self->sizes[d]; }
  }
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, nd, index->sizes, idx);
    int64_t k = load_int(index, offset_of(index, idx));
    int64_t so = offset_of(src, idx);
    if (nd) idx[dim] = k;
    if (flt) {
      int64_t l = 0;
      for (int d = 0; d < nd; ++d) l += idx[d] * lstr[d];
      acc[(size_t)l] += load_flt(src, so);
      touched[(size_t)l] = 1;
    } else {
      int64_t d = offset_of(self, idx);
      if (self->dtype == ORC_BOOL) store_int(self, d, load_int(self, d) | load_int(src, so));
      else store_int(self, d, (int64_t)((uint64_t)load_int(self, d) + (uint64_t)load_int(src, so)));
    }
  }
  if (flt) {
    for (int64_t l = 0; l < nself; ++l) {
      if (!touched[(size_t)l]) continue;               // untouched elements keep their bits
      int64_t idx[ORC_MAX_DIMS] = {0};
      unravel(l, nd, self->sizes, idx);
      int64_t d = offset_of(self, idx);
      store_flt(self, d, load_flt(self, d) + acc[(size_t)l]);
    }
  }
  return ORC_OK;
}

// scatter_reduce_ (in place on self): every position p of index sends src[p] to self[p with coordinate dim =
// index[p]], where the values that arrive are combined with the element's own value by `reduce`:
//   0 sum, 1 prod, 2 mean, 3 amax, 4 amin.
// include_self == 0: an element that receives at least one value starts from the values alone (its old content is
// dropped); elements that receive nothing always keep their bits.  Shapes and dtypes as scatter_add_.  bool: sum and
// amax are OR, prod and amin are AND, mean is refused.
//   sum / prod : integers wrap; floats accumulate in binary64 in position order, one rounding.
//   mean       : (sum of the values [+ self]) / (their number [+ 1]); integers divide rounding toward -infinity;
//                floats in binary64, one rounding.
//   amax / amin: the largest / smallest; a NaN among the values (or in self when it is included) gives NaN.
int orc_scatter_reduce(const orc_tensor* self, int64_t dim, const orc_tensor* index, const orc_tensor* src, int reduce,
                       int include_self) {
  int rc;
  if ((rc = check_tensor(self)) || (rc = check_tensor(index)) || (rc = check_tensor(src))) return rc;
  if (!index_dtype_ok(index->dtype)) return ORC_ERR_DTYPE;
  if (self->dtype != src->dtype) return ORC_ERR_DTYPE;
  if (reduce < 0 || reduce > 4) return ORC_ERR_SCALAR;
  if (self->dtype == ORC_BOOL && reduce == 2) return ORC_ERR_DTYPE;   // no mean of bools
  if (index->ndim != self->ndim || src->ndim != self->ndim) return ORC_ERR_SHAPE;
  const int nd = self->ndim;
  int lim = nd == 0 ? 1 : nd;
  if (dim < -lim || dim >= lim) return ORC_ERR_DIM;
  if (dim < 0) dim += lim;
  for (int d = 0; d < nd; ++d) {
    if (index->sizes[d] > src->sizes[d]) return ORC_ERR_SHAPE;
    if (d != dim && index->sizes[d] > self->sizes[d]) return ORC_ERR_SHAPE;
  }
  const int64_t n = numel(index);
  if (n == 0) return ORC_OK;
  const int64_t extent = nd == 0 ? 1 : self->sizes[dim];
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, nd, index->sizes, idx);
    int64_t k = load_int(index, offset_of(index, idx));
    if (k < 0 || k >= extent) return ORC_ERR_INDEX;
  }
  const bool flt = is_float(self->dtype);
  const int64_t nself = numel(self);
  int64_t lstr[ORC_MAX_DIMS];
  { int64_t st = 1; for (int d = nd - 1; d >= 0; --d) { lstr[d] = st; st *= self->sizes[d]; } }
  // per destination element (logical index): number of values, and their running combination
  std::vector<int64_t> cnt((size_t)nself, 0);
  std::vector<double> accd;
  std::vector<int64_t> acci;
  if (flt) accd.assign((size_t)nself, 0.0); else acci.assign((size_t)nself, 0);
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, nd, index->sizes, idx);
    const int64_t k = load_int(index, offset_of(index, idx));
    const int64_t so = offset_of(src, idx);
    if (nd) idx[dim] = k;
    int64_t l = 0;
    for (int d = 0; d < nd; ++d) l += idx[d] * lstr[d];
    const bool first = cnt[(size_t)l]++ == 0;
    if (flt) {
      const double v = load_flt(src, so);
      double& a = accd[(size_t)l];
      if (first) a = v;
      else switch (reduce) {
        case 0: case 2: a += v; break;
        case 1: a *= v; break;
        case 3: a = (std::isnan(a) || std::isnan(v)) ? kNaN : (v > a ? v : a); break;
        case 4: a = (std::isnan(a) || std::isnan(v)) ? kNaN : (v < a ? v : a); break;
      }
    } else {
      const int64_t v = load_int(src, so);
      int64_t& a = acci[(size_t)l];
      if (first) a = v;
      else switch (reduce) {
        case 0: case 2: a = (int64_t)((uint64_t)a + (uint64_t)v); break;
        case 1: a = (int64_t)((uint64_t)a * (uint64_t)v); break;
        case 3: a = v > a ? v : a; break;
        case 4: a = v < a ? v : a; break;
      }
      if (self->dtype == ORC_I32) a = (int64_t)(int32_t)(uint32_t)(uint64_t)a;      // int32 arithmetic wraps at 32 bits
    }
  }
  for (int64_t l = 0; l < nself; ++l) {
    if (!cnt[(size_t)l]) continue;
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(l, nd, self->sizes, idx);
    const int64_t d_o = offset_of(self, idx);
    const int64_t c = cnt[(size_t)l] + (include_self ? 1 : 0);
    if (flt) {
      double a = accd[(size_t)l];
      if (include_self) {
        const double s0 = load_flt(self, d_o);
        switch (reduce) {
          case 0: case 2: a += s0; break;
          case 1: a *= s0; break;
          case 3: a = (std::isnan(a) || std::isnan(s0)) ? kNaN : (s0 > a ? s0 : a); break;
          case 4: a = (std::isnan(a) || std::isnan(s0)) ? kNaN : (s0 < a ? s0 : a); break;
        }
      }
      if (reduce == 2) a /= (double)c;
      store_flt(self, d_o, a);
    } else {
      int64_t a = acci[(size_t)l];
      if (include_self) {
        const int64_t s0 = load_int(self, d_o);
        switch (reduce) {
          case 0: case 2: a = (int64_t)((uint64_t)a + (uint64_t)s0); break;
          case 1: a = (int64_t)((uint64_t)a * (uint64_t)s0); break;
          case 3: a = s0 > a ? s0 : a; break;
          case 4: a = s0 < a ? s0 : a; break;
        }
        if (self->dtype == ORC_I32) a = (int64_t)(int32_t)(uint32_t)(uint64_t)a;
      }
      if (reduce == 2) {                                 // floor division
        int64_t q = a / c;
        if ((a % c != 0) && ((a < 0) != (c < 0))) --q;
        a = q;
      }
      store_int(self, d_o, a);
    }
  }
  return ORC_OK;
}

// index_put_ (in place on self): `nidx` index tensors address the first nidx dims of self.  They broadcast together
// to a shape I; values has shape I + self.shape[nidx:] (or broadcasts to it).  For every position p of I and every
// coordinate r of the remaining dims: self[idx_0[p], ..., idx_{k-1}[p], r] = values[p, r], or += when accumulate.
// Negative indices count from the end.  accumulate: integers wrap (bool: OR); floats gather each destination's
// values in position order in binary64, add the old content, round once.  Without accumulate, when several positions
// name one destination the LAST in position order is kept here (the operator itself leaves the winner undefined).
int orc_index_put(const orc_tensor* self, const orc_tensor* const* indices, int32_t nidx, const orc_tensor* values,
                  int accumulate) {
  int rc;
  if ((rc = check_tensor(self)) || (rc = check_tensor(values))) return rc;
  if (nidx < 1 || nidx > self->ndim) return ORC_ERR_DIM;
  for (int j = 0; j < nidx; ++j) {
    if (!indices || (rc = check_tensor(indices[j]))) return rc ? rc : ORC_ERR_NULL;
    if (!index_dtype_ok(indices[j]->dtype)) return ORC_ERR_DTYPE;
  }
  if (values->dtype != self->dtype) return ORC_ERR_DTYPE;
  int ind;
  int64_t ishape[ORC_MAX_DIMS];
  if ((rc = broadcast_shapes(indices, nidx, &ind, ishape))) return rc;
  const int rest = self->ndim - nidx;
  if (ind + rest > ORC_MAX_DIMS) return ORC_ERR_NDIM;
  // the full shape values must broadcast to: I + remaining dims of self
  int64_t vshape[ORC_MAX_DIMS];
  const int vnd = ind + rest;
  for (int d = 0; d < ind; ++d) vshape[d] = ishape[d];
  for (int d = 0; d < rest; ++d) vshape[ind + d] = self->sizes[nidx + d];
  if (values->ndim > vnd) return ORC_ERR_SHAPE;
  for (int d = 0; d < values->ndim; ++d) {
    const int64_t vs = values->sizes[d], ts = vshape[vnd - values->ndim + d];
    if (vs != ts && vs != 1) return ORC_ERR_SHAPE;
  }
  int64_t n = 1;
  for (int d = 0; d < vnd; ++d) n *= vshape[d];
  // validate (and wrap) every index first
  int64_t npos = 1;
  for (int d = 0; d < ind; ++d) npos *= ishape[d];
  for (int64_t p = 0; p < npos; ++p) {
    int64_t pidx[ORC_MAX_DIMS] = {0};
    unravel(p, ind, ishape, pidx);
    for (int j = 0; j < nidx; ++j) {
      const int64_t k = load_int(indices[j], bcast_offset(indices[j], ind, pidx));
      if (k < -self->sizes[j] || k >= self->sizes[j]) return ORC_ERR_INDEX;
    }
  }
  const bool flt = is_float(self->dtype);
  const int64_t nself = numel(self);
  int64_t lstr[ORC_MAX_DIMS];
  { int64_t st = 1; for (int d = self->ndim - 1; d >= 0; --d) { lstr[d] = st; st *= self->sizes[d]; } }
  std::vector<double> acc;
  std::vector<uint8_t> touched;
  if (flt && accumulate) { acc.assign((size_t)nself, 0.0); touched.assign((size_t)nself, 0); }
  const int es = esize(self->dtype);
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t vidx[ORC_MAX_DIMS] = {0};
    unravel(lin, vnd, vshape, vidx);
    int64_t sidx[ORC_MAX_DIMS] = {0};
    for (int j = 0; j < nidx; ++j) {
      int64_t k = load_int(indices[j], bcast_offset(indices[j], ind, vidx));
      sidx[j] = k < 0 ? k + self->sizes[j] : k;
    }
    for (int d = 0; d < rest; ++d) sidx[nidx + d] = vidx[ind + d];
    const int64_t d_o = offset_of(self, sidx);
    const int64_t vo = bcast_offset(values, vnd, vidx);
    if (!accumulate) {
      std::memcpy(mptr(self, d_o), cptr(values, vo), es);
    } else if (flt) {
      int64_t l = 0;
      for (int d = 0; d < self->ndim; ++d) l += sidx[d] * lstr[d];
      acc[(size_t)l] += load_flt(values, vo);
      touched[(size_t)l] = 1;
    } else if (self->dtype == ORC_BOOL) {
      store_int(self, d_o, load_int(self, d_o) | load_int(values, vo));
    } else {
      store_int(self, d_o, (int64_t)((uint64_t)load_int(self, d_o) + (uint64_t)load_int(values, vo)));
    }
  }
  if (flt && accumulate) {
    for (int64_t l = 0; l < nself; ++l) {
      if (!touched[(size_t)l]) continue;
      int64_t idx[ORC_MAX_DIMS] = {0};
      unravel(l, self->ndim, self->sizes, idx);
      const int64_t d_o = offset_of(self, idx);
      store_flt(self, d_o, load_flt(self, d_o) + acc[(size_t)l]);
    }
  }
  return ORC_OK;
}

// index_add_ (in place on self): for every i, self[..., index[i], ...] += alpha * source[..., i, ...] along `dim`.
// index is 1-D (or 0-dim) int32 / int64 with source.size(dim) entries in [0, self.size(dim)); source has self's
// shape except along dim; both have the same dtype.  Integers: exact wrapping arithmetic, alpha must be integral;
// bool: self OR (alpha != 0 AND source).  Floating dtypes: the products alpha * source are accumulated per destination element in
// binary64 in index order, the initial value of self is added, one rounding.
int orc_index_add(const orc_tensor* self, int64_t dim, const orc_tensor* index, const orc_tensor* source, double alpha_f,
                  int64_t alpha_i, int alpha_is_int) {
  int rc;
  if ((rc = check_tensor(self)) || (rc = check_tensor(index)) || (rc = check_tensor(source))) return rc;
  if (!index_dtype_ok(index->dtype)) return ORC_ERR_DTYPE;
  if (self->dtype != source->dtype) return ORC_ERR_DTYPE;
  if (index->ndim > 1 || source->ndim != self->ndim) return ORC_ERR_SHAPE;
  const int nd = self->ndim;
  int lim = nd == 0 ? 1 : nd;
  if (dim < -lim || dim >= lim) return ORC_ERR_DIM;
  if (dim < 0) dim += lim;
  const int64_t ni = numel(index);
  if ((nd == 0 ? 1 : source->sizes[dim]) != ni) return ORC_ERR_SHAPE;
  for (int d = 0; d < nd; ++d)
    if (d != dim && source->sizes[d] != self->sizes[d]) return ORC_ERR_SHAPE;
  const bool flt = is_float(self->dtype);
  if (!flt && !alpha_is_int) return ORC_ERR_SCALAR;
  const int64_t extent = nd == 0 ? 1 : self->sizes[dim];
  const int64_t istride = index->ndim ? index->strides[0] : 0;
  for (int64_t i = 0; i < ni; ++i) {
    int64_t k = load_int(index, i * istride);
    if (k < 0 || k >= extent) return ORC_ERR_INDEX;      // checked first: nothing is written on error
  }
  const double alpha = alpha_is_int ? (double)alpha_i : alpha_f;
  // walk source in logical order: for one destination element the contributions then arrive in index order
  const int64_t nself = numel(self), nsrc = numel(source);
  std::vector<double> acc;
  std::vector<uint8_t> touched;
  int64_t lstr[ORC_MAX_DIMS];                          // row-major strides of self's logical shape
  if (flt) {
    acc.assign((size_t)nself, 0.0);
    touched.assign((size_t)nself, 0);
    int64_t st = 1;
    for (int d = nd - 1; d >= 0; --d) { lstr[d] = st; st *= self->sizes[d]; }
  }
  for (int64_t lin = 0; lin < nsrc; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, nd, source->sizes, idx);
    const int64_t so = offset_of(source, idx);
    const int64_t i = nd ? idx[dim] : 0;
    if (nd) idx[dim] = load_int(index, i * istride);
    if (flt) {
      int64_t l = 0;
      for (int d = 0; d < nd; ++d) l += idx[d] * lstr[d];
      acc[(size_t)l] += alpha * load_flt(source, so);
      touched[(size_t)l] = 1;
    } else {
      const int64_t d_o = offset_of(self, idx);
      if (self->dtype == ORC_BOOL) store_int(self, d_o, load_int(self, d_o) | ((alpha_i != 0) & load_int(source, so)));
      else store_int(self, d_o, (int64_t)((uint64_t)load_int(self, d_o) + (uint64_t)alpha_i * (uint64_t)load_int(source, so)));
    }
  }
  if (flt) {
    for (int64_t l = 0; l < nself; ++l) {
      if (!touched[(size_t)l]) continue;               // untouched elements keep their bits
      int64_t idx[ORC_MAX_DIMS] = {0};
      unravel(l, nd, self->sizes, idx);
      const int64_t d_o = offset_of(self, idx);
      store_flt(self, d_o, load_flt(self, d_o) + acc[(size_t)l]);
    }
  }
  return ORC_OK;
}

// take(input, index): out[p] = input viewed as a 1-D tensor in logical (row-major) order, at index[p]; negative
// indices count from the end.  out has index's shape and input's dtype.  An index outside [-n, n) is an error.
int orc_take(const orc_tensor* out, const orc_tensor* input, const orc_tensor* index) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(input)) || (rc = check_tensor(index))) return rc;
  if (!index_dtype_ok(index->dtype)) return ORC_ERR_DTYPE;
  if (out->dtype != input->dtype) return ORC_ERR_DTYPE;
  if (!same_shape(out, index->ndim, index->sizes)) return ORC_ERR_SHAPE;
  const int64_t n = numel(input), m = numel(index);
  const int es = esize(input->dtype);
  for (int pass = 0; pass < 2; ++pass) {                 // pass 0 validates, pass 1 writes
    for (int64_t lin = 0; lin < m; ++lin) {
      int64_t idx[ORC_MAX_DIMS] = {0};
      unravel(lin, index->ndim, index->sizes, idx);
      int64_t k = load_int(index, offset_of(index, idx));
      if (k < -n || k >= n) return ORC_ERR_INDEX;
      if (!pass) continue;
      if (k < 0) k += n;
      int64_t sidx[ORC_MAX_DIMS] = {0};
      unravel(k, input->ndim, input->sizes, sidx);
      std::memcpy(mptr(out, offset_of(out, idx)), cptr(input, offset_of(input, sidx)), es);
    }
  }
  return ORC_OK;
}

// searchsorted(sorted_sequence, values, right) / bucketize: for every value the index at which it would be inserted
// into its sequence so that the order is kept - the first position whose element is >= v (left) or > v (right).
// A 1-D sequence serves every value; otherwise the sequence has the values' rank and leading dims and each row of
// values is searched in the matching row.  The index is found by bisection of [0, n) with the midpoint
// start + (end - start) / 2, moving right while !(element >= v) (left) or !(element > v) (right): on a sorted
// sequence without NaN this is the count of elements below v (at most v); a NaN value lands at n, and on other
// inputs the result is whatever these steps give.  Both dtypes must be equal and not bool; out is int64 or int32.
int orc_searchsorted(const orc_tensor* out, const orc_tensor* seq, const orc_tensor* values, int right) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(seq)) || (rc = check_tensor(values))) return rc;
  if (seq->dtype != values->dtype || seq->dtype == ORC_BOOL) return ORC_ERR_DTYPE;
  if (out->dtype != ORC_I64 && out->dtype != ORC_I32) return ORC_ERR_DTYPE;
  if (seq->ndim < 1) return ORC_ERR_NDIM;
  if (seq->ndim != 1) {
    if (seq->ndim != values->ndim) return ORC_ERR_SHAPE;
    for (int d = 0; d + 1 < seq->ndim; ++d)
      if (seq->sizes[d] != values->sizes[d]) return ORC_ERR_SHAPE;
  }
  if (!same_shape(out, values->ndim, values->sizes)) return ORC_ERR_SHAPE;
  const int64_t m = numel(values), n = seq->sizes[seq->ndim - 1];
  const bool flt = is_float(seq->dtype);
  for (int64_t lin = 0; lin < m; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, values->ndim, values->sizes, idx);
    const Val v = load_as(values, offset_of(values, idx), values->dtype);
    int64_t sidx[ORC_MAX_DIMS] = {0};
    if (seq->ndim != 1)
      for (int d = 0; d + 1 < seq->ndim; ++d) sidx[d] = idx[d];
    int64_t start = 0, end = n;
    while (start < end) {
      const int64_t mid = start + (end - start) / 2;
      sidx[seq->ndim - 1] = mid;
      const Val e = load_as(seq, offset_of(seq, sidx), seq->dtype);
      const bool stop = flt ? (right ? e.f > v.f : e.f >= v.f) : (right ? e.i > v.i : e.i >= v.i);
      if (!stop) start = mid + 1;
      else end = mid;
    }
    store_int(out, offset_of(out, idx), start);
  }
  return ORC_OK;
}

// masked_select(x, mask): the elements of x (broadcast with the bool mask) where the mask is true, in logical
// (row-major) order of the broadcast shape.  `out` is a 1-D buffer of x's dtype with room for them (its first
// *count elements are written; a smaller buffer is a shape error and nothing is written).
int orc_masked_select(const orc_tensor* out, const orc_tensor* x, const orc_tensor* mask, int64_t* count) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x)) || (rc = check_tensor(mask))) return rc;
  if (mask->dtype != ORC_BOOL || out->dtype != x->dtype) return ORC_ERR_DTYPE;
  if (out->ndim != 1) return ORC_ERR_SHAPE;
  const orc_tensor* ops[2] = {x, mask};
  int nd;
  int64_t sizes[ORC_MAX_DIMS];
  if ((rc = broadcast_shapes(ops, 2, &nd, sizes))) return rc;
  int64_t n = 1;
  for (int d = 0; d < nd; ++d) n *= sizes[d];
  int64_t c = 0;
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, sizes, idx);
    c += load_int(mask, bcast_offset(mask, nd, idx)) != 0;
  }
  if (count) *count = c;
  if (out->sizes[0] < c) return ORC_ERR_SHAPE;
  const int es = esize(x->dtype);
  int64_t w = 0;
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    unravel(lin, nd, sizes, idx);
    if (!load_int(mask, bcast_offset(mask, nd, idx))) continue;
    std::memcpy(mptr(out, w * out->strides[0]), cptr(x, bcast_offset(x, nd, idx)), es);
    ++w;
  }
  return ORC_OK;
}

// nonzero(x): the multi-indices of the elements that are not zero (a NaN is not zero; -0.0 is zero), in logical
// (row-major) order, one row of x.ndim int64 coordinates each.  `out` is a 2-D int64 buffer [capacity, x.ndim];
// its first *count rows are written (a smaller buffer is a shape error and nothing is written).
int orc_nonzero(const orc_tensor* out, const orc_tensor* x, int64_t* count) {
  int rc;
  if ((rc = check_tensor(out)) || (rc = check_tensor(x))) return rc;
  if (out->dtype != ORC_I64) return ORC_ERR_DTYPE;
  if (out->ndim != 2 || out->sizes[1] != x->ndim) return ORC_ERR_SHAPE;
  const int64_t n = numel(x);
  auto is_nz = [&](int64_t off) { return is_float(x->dtype) ? !(load_flt(x, off) == 0.0) : load_int(x, off) != 0; };
  int64_t c = 0;
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, x->ndim, x->sizes, idx);
    c += is_nz(offset_of(x, idx));
  }
  if (count) *count = c;
  if (out->sizes[0] < c) return ORC_ERR_SHAPE;
  int64_t w = 0;
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS] = {0};
    unravel(lin, x->ndim, x->sizes, idx);
    if (!is_nz(offset_of(x, idx))) continue;
    for (int d = 0; d < x->ndim; ++d) store_int(out, w * out->strides[0] + d * out->strides[1], idx[d]);
    ++w;
  }
  return ORC_OK;
}

// Test hooks for the format codecs: encode a binary64 value into `dtype`
// (F16 / BF16 / F32) with one rounding, and decode a bit pattern exactly.
uint32_t orc_encode(double v, int dtype) {
  if (dtype == ORC_F16) return double_to_f16(v);
  if (dtype == ORC_BF16) return double_to_bf16(v);
  float f = (float)v;
  uint32_t b;
  std::memcpy(&b, &f, 4);
  return b;
}
double orc_decode(uint32_t bits, int dtype) {
  if (dtype == ORC_F16) return f16_to_double((uint16_t)bits);
  if (dtype == ORC_BF16) return bf16_to_double((uint16_t)bits);
  float f;
  std::memcpy(&f, &bits, 4);
  return (double)f;
}

// Number of OpenMP threads a parallel region will use (for reporting).
int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// Sets the number of OpenMP threads later parallel regions use (for timing the
// same code on one core and on all of them; results do not depend on it).
void orc_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

}  // extern "C"
