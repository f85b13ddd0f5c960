// Host-side validation, type promotion, broadcasting, overlap rules and the
// result-inference entry points.  No device code here.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>

#include "common.h"

namespace tx {

namespace {
thread_local char g_err[512] = "";
thread_local const char* g_path = "";
thread_local std::string g_forced;
}  // namespace

const char* dtype_name(int dt) {
  static const char* names[] = {"bool", "int32", "int64", "float16", "bfloat16", "float32"};
  return dtype_valid(dt) ? names[dt] : "invalid";
}

tx_status fail(tx_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void set_path(const char* name) { g_path = name; }
const char* forced_path() { return g_forced.c_str(); }

tx_status check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TX_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
  return TX_OK;
}

tx_status check_tensor(const tx_tensor* t, const char* name) {
  if (!t) return fail(TX_ERR_NULL, "%s: null descriptor", name);
  if (t->ndim < 0 || t->ndim > TX_MAX_DIMS) return fail(TX_ERR_NDIM, "%s: ndim %d", name, t->ndim);
  if (!dtype_valid(t->dtype)) return fail(TX_ERR_DTYPE, "%s: dtype code %d", name, t->dtype);
  for (int d = 0; d < t->ndim; ++d) {
    if (t->sizes[d] < 0) return fail(TX_ERR_SHAPE, "%s: negative size", name);
    if (t->strides[d] < 0) return fail(TX_ERR_SHAPE, "%s: negative stride", name);
  }
  if (numel(t) > 0 && !t->data) return fail(TX_ERR_NULL, "%s: null data", name);
  return TX_OK;
}

bool same_sizes(const tx_tensor* t, int nd, const int64_t* sizes) {
  if (t->ndim != nd) return false;
  for (int d = 0; d < nd; ++d)
    if (t->sizes[d] != sizes[d]) return false;
  return true;
}

tx_status wrap_dim(int64_t dim, int nd, int* out) {
  int lim = nd == 0 ? 1 : nd;
  if (dim < -lim || dim >= lim) return fail(TX_ERR_DIM, "dim %lld out of range for rank %d", (long long)dim, nd);
  *out = (int)(dim < 0 ? dim + lim : dim);
  return TX_OK;
}

int promote2(int a, int b) {
  if (a == b) return a;
  int ca = dtype_category(a), cb = dtype_category(b);
  if (ca != cb) return ca > cb ? a : b;
  if (ca == 1) return TX_I64;
  return TX_F32;   // two different float types: anything with fp32, or fp16 with bf16
}

int result_type(const tx_tensor* const* ops, int n) {
  int dimd = -1, zero = -1;
  for (int i = 0; i < n; ++i) {
    int& g = ops[i]->ndim >= 1 ? dimd : zero;
    g = g < 0 ? ops[i]->dtype : promote2(g, ops[i]->dtype);
  }
  if (dimd < 0) return zero;
  if (zero < 0) return dimd;
  return dtype_category(dimd) >= dtype_category(zero) ? dimd : zero;
}

tx_status broadcast_shapes(const tx_tensor* const* ops, int n, int* ndim, int64_t* sizes) {
  int nd = 0;
  for (int i = 0; i < n; ++i) nd = std::max(nd, (int)ops[i]->ndim);
  for (int d = 0; d < nd; ++d) sizes[d] = 1;
  for (int i = 0; i < n; ++i) {
    int shift = nd - ops[i]->ndim;
    for (int d = 0; d < ops[i]->ndim; ++d) {
      int64_t s = ops[i]->sizes[d];
      int64_t& o = sizes[d + shift];
      if (s == o) continue;
      if (o == 1) o = s;
      else if (s != 1)
        return fail(TX_ERR_SHAPE, "operands are not broadcastable (dim %d: %lld vs %lld)", d + shift, (long long)o,
                    (long long)s);
    }
  }
  *ndim = nd;
  return TX_OK;
}

void byte_extent(const tx_tensor* t, uintptr_t* lo, uintptr_t* hi) {
  uintptr_t base = (uintptr_t)t->data;
  *lo = *hi = base;
  if (numel(t) == 0) return;
  int64_t last = 0;
  for (int d = 0; d < t->ndim; ++d) last += (t->sizes[d] - 1) * t->strides[d];
  *hi = base + (uintptr_t)(last + 1) * dtype_size(t->dtype);
}

bool no_internal_overlap(const tx_tensor* t) {
  // sort dims with size > 1 by stride; every stride must clear the span of all smaller ones
  int64_t st[TX_MAX_DIMS], sz[TX_MAX_DIMS];
  int n = 0;
  for (int d = 0; d < t->ndim; ++d) {
    if (t->sizes[d] == 0) return true;
    if (t->sizes[d] > 1) { st[n] = t->strides[d]; sz[n] = t->sizes[d]; ++n; }
  }
  for (int i = 1; i < n; ++i)
    for (int j = i; j > 0 && st[j] < st[j - 1]; --j) { std::swap(st[j], st[j - 1]); std::swap(sz[j], sz[j - 1]); }
  int64_t span = 0;   // largest offset reachable with the dims seen so far
  for (int i = 0; i < n; ++i) {
    if (st[i] <= span) return false;
    span += (sz[i] - 1) * st[i];
  }
  return true;
}

bool partial_overlap(const tx_tensor* out, const tx_tensor* in) {
  if (numel(out) == 0 || numel(in) == 0) return false;
  uintptr_t olo, ohi, ilo, ihi;
  byte_extent(out, &olo, &ohi);
  byte_extent(in, &ilo, &ihi);
  if (ohi <= ilo || ihi <= olo) return false;
  // identical view: in-place use
  if (out->data == in->data && out->dtype == in->dtype && out->ndim == in->ndim) {
    bool same = true;
    for (int d = 0; d < out->ndim; ++d)
      if (out->sizes[d] != in->sizes[d] || (out->sizes[d] > 1 && out->strides[d] != in->strides[d])) same = false;
    if (same) return false;
  }
  return true;
}

}  // namespace tx

using namespace tx;

extern "C" {

const char* tx_strerror(tx_status s) {
  switch (s) {
    case TX_OK: return "ok";
    case TX_ERR_NULL: return "null pointer";
    case TX_ERR_NDIM: return "bad ndim";
    case TX_ERR_DTYPE: return "dtype not accepted";
    case TX_ERR_SHAPE: return "shape mismatch";
    case TX_ERR_DIM: return "bad dim";
    case TX_ERR_OVERLAP: return "memory overlap";
    case TX_ERR_EMPTY_REDUCTION: return "reduction over an empty extent";
    case TX_ERR_SCALAR: return "scalar not representable in the result dtype";
    case TX_ERR_WORKSPACE: return "workspace too small";
    case TX_ERR_INDEX: return "index out of range";
    case TX_ERR_LAUNCH: return "kernel launch failed";
    case TX_ERR_UNSUPPORTED: return "unsupported";
  }
  return "unknown status";
}
const char* tx_last_error(void) { return g_err; }
const char* tx_last_path(void) { return g_path; }
void tx_force_path(const char* name) { g_forced = name ? name : ""; }

int32_t tx_infer_unary_dtype(int op, int32_t in) {
  if (!dtype_valid(in)) return fail(TX_ERR_DTYPE, "unary: dtype code %d", in);
  switch (op) {
    case TX_NEG:
    case TX_ABS:
      if (in == TX_BOOL) return fail(TX_ERR_DTYPE, "neg/abs do not take bool");
      return in;
    case TX_EXP: case TX_LOG: case TX_SQRT: case TX_SIGMOID: case TX_TANH: case TX_LOG1P: case TX_EXPM1:
      return dtype_is_float(in) ? in : TX_F32;
    case TX_GELU_ERF: case TX_LOGSIGMOID:
      if (!dtype_is_float(in)) return fail(TX_ERR_DTYPE, "gelu / logsigmoid take floating dtypes only");
      return in;
    case TX_LOGICAL_NOT: case TX_ISNAN: case TX_ISINF: case TX_ISFINITE:
      return TX_BOOL;
    case TX_SIN: case TX_COS: case TX_EXP2: case TX_LOG2: case TX_LOG10: case TX_RSQRT: case TX_RECIPROCAL:
      return dtype_is_float(in) ? in : TX_F32;
    case TX_SILU:
      if (!dtype_is_float(in)) return fail(TX_ERR_DTYPE, "silu takes floating dtypes only");
      return in;
    case TX_SQUARE:
      return in == TX_BOOL ? TX_I64 : in;
    case TX_SIGN:
      return in;
    case TX_FLOOR: case TX_CEIL: case TX_TRUNC: case TX_ROUND:
      if (in == TX_BOOL) return fail(TX_ERR_DTYPE, "floor / ceil / trunc / round do not take bool");
      return in;
    case TX_BITWISE_NOT:
      if (dtype_is_float(in)) return fail(TX_ERR_DTYPE, "bitwise_not takes integer and bool dtypes only");
      return in;
    case TX_TAN: case TX_ASIN: case TX_ACOS: case TX_ATAN: case TX_SINH: case TX_COSH: case TX_ASINH: case TX_ACOSH:
    case TX_ATANH: case TX_ERF: case TX_ERFC:
      return dtype_is_float(in) ? in : TX_F32;
    case TX_RELU:
      if (in == TX_BOOL) return fail(TX_ERR_DTYPE, "relu does not take bool");
      return in;
    case TX_FRAC: case TX_HARDSWISH: case TX_HARDSIGMOID: case TX_MISH:
      if (!dtype_is_float(in)) return fail(TX_ERR_DTYPE, "frac / hardswish / hardsigmoid / mish take floating dtypes only");
      return in;
    case TX_SIGNBIT:
      return TX_BOOL;
  }
  return fail(TX_ERR_DTYPE, "unknown unary op %d", op);
}

tx_status tx_infer_binary(int op, const tx_tensor* a, const tx_tensor* b, int32_t* dtype, int32_t* ndim,
                          int64_t* sizes) {
  if (!a || !b) return fail(TX_ERR_NULL, "infer_binary: null descriptor");
  if (a->ndim < 0 || a->ndim > TX_MAX_DIMS || b->ndim < 0 || b->ndim > TX_MAX_DIMS)
    return fail(TX_ERR_NDIM, "infer_binary: bad ndim");
  if (!dtype_valid(a->dtype) || !dtype_valid(b->dtype)) return fail(TX_ERR_DTYPE, "infer_binary: bad dtype code");
  if (op < TX_ADD || op > TX_TRUNC_DIVIDE) return fail(TX_ERR_DTYPE, "unknown binary op %d", op);
  const tx_tensor* ops[2] = {a, b};
  int common = result_type(ops, 2);
  int res = common;
  if (op == TX_DIV && !dtype_is_float(common)) res = TX_F32;
  if (op == TX_EQ || (op >= TX_NE && op <= TX_LOGICAL_XOR)) res = TX_BOOL;
  if (op == TX_POW && common == TX_BOOL) return fail(TX_ERR_DTYPE, "pow does not take two bool operands");
  if (op >= TX_BITWISE_AND && op <= TX_BITWISE_XOR && dtype_is_float(common))
    return fail(TX_ERR_DTYPE, "bitwise operators take integer and bool dtypes only");
  if (op == TX_ATAN2 && !dtype_is_float(common)) res = TX_F32;
  if ((op == TX_FMOD || op == TX_REMAINDER || op == TX_FLOOR_DIVIDE || op == TX_TRUNC_DIVIDE) && common == TX_BOOL)
    return fail(TX_ERR_DTYPE, "fmod / remainder / floor_divide / trunc_divide do not take two bool operands");
  if ((op == TX_HYPOT || op == TX_LOGADDEXP || op == TX_LOGADDEXP2 || op == TX_NEXTAFTER) && !dtype_is_float(common))
    return fail(TX_ERR_DTYPE, "hypot / logaddexp / logaddexp2 / nextafter need a floating operand");
  if ((op == TX_COPYSIGN || op == TX_XLOGY) && !dtype_is_float(common)) res = TX_F32;
  if (op == TX_HEAVISIDE && a->dtype != b->dtype) return fail(TX_ERR_DTYPE, "heaviside takes two operands of one dtype");
  if (op >= TX_GCD && op <= TX_SHIFT_RIGHT && (dtype_is_float(common) || common == TX_BOOL))
    return fail(TX_ERR_DTYPE, "gcd / lcm / shifts take int32 / int64 (a bool with an integer promotes)");
  if (op == TX_SUB && (a->dtype == TX_BOOL || b->dtype == TX_BOOL))
    return fail(TX_ERR_DTYPE, "sub does not take bool operands");
  int nd;
  int64_t s[TX_MAX_DIMS];
  tx_status rc = broadcast_shapes(ops, 2, &nd, s);
  if (rc) return rc;
  if (dtype) *dtype = res;
  if (ndim) *ndim = nd;
  if (sizes) std::copy(s, s + nd, sizes);
  return TX_OK;
}

int32_t tx_infer_clamp_dtype(int32_t x_dtype, int has_lo, int lo_is_int, int has_hi, int hi_is_int) {
  if (!dtype_valid(x_dtype)) return fail(TX_ERR_DTYPE, "clamp: dtype code %d", x_dtype);
  if (x_dtype == TX_BOOL) return fail(TX_ERR_DTYPE, "clamp does not take bool");
  if (!has_lo && !has_hi) return fail(TX_ERR_SCALAR, "clamp needs at least one bound");
  if (dtype_is_float(x_dtype)) return x_dtype;
  return ((has_lo && !lo_is_int) || (has_hi && !hi_is_int)) ? TX_F32 : x_dtype;
}

tx_status tx_infer_where(const tx_tensor* x, const tx_tensor* y, int32_t* dtype) {
  if (!x || !y) return fail(TX_ERR_NULL, "infer_where: null descriptor");
  const tx_tensor* ops[2] = {x, y};
  if (dtype) *dtype = result_type(ops, 2);
  return TX_OK;
}

}  // extern "C"
