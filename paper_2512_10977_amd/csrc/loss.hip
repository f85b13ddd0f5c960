// binary_cross_entropy and the regression losses (mse, l1, smooth_l1, huber):
// the elementwise form on the operand iterator's paths, and the dispatch of the
// sum / mean forms (fused single pass when the operands can be read linearly,
// otherwise the losses are formed in the workspace first and summed from there).
#include "ew_impl.h"
#include "loss.h"

namespace tx {
namespace {

template <bool HAS_W> struct BceF32 {
  using Out = float; using In0 = float; using In1 = float; using In2 = typename std::conditional<HAS_W, float, void>::type;
  static constexpr int NIN = HAS_W ? 3 : 2;
  __device__ __forceinline__ float operator()(float x, float t) const { return bce_term(x, t); }
  __device__ __forceinline__ float operator()(float x, float t, float w) const { return bce_term(x, t) * w; }
};
// half types, or a weight of another floating dtype: values converted on load, the loss rounded once on store
template <bool HAS_W> struct BceDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>;
  using In2 = typename std::conditional<HAS_W, Dyn<float>, void>::type;
  static constexpr int NIN = HAS_W ? 3 : 2;
  __device__ __forceinline__ float operator()(float x, float t) const { return bce_term(x, t); }
  __device__ __forceinline__ float operator()(float x, float t, float w) const { return bce_term(x, t) * w; }
};

tx_status bce_elementwise(const tx_tensor* out, const tx_tensor* x, const tx_tensor* t, const tx_tensor* w, hipStream_t s) {
  const tx_tensor* ops[4] = {out, x, t, w};
  Iter it;
  iter_build(&it, x->ndim, x->sizes, ops, w ? 4 : 3);
  const bool f32 = x->dtype == TX_F32 && (!w || w->dtype == TX_F32);
  if (w) return f32 ? launch_ew(it, BceF32<true>{}, s) : launch_ew(it, BceDyn<true>{}, s);
  return f32 ? launch_ew(it, BceF32<false>{}, s) : launch_ew(it, BceDyn<false>{}, s);
}

// regression losses, one term: see loss_term in norm.hip for the forms (kind 1 mse, 2 l1, 3 smooth_l1, 4 huber)
__device__ __forceinline__ float regression_term(int kind, float x, float t, float p, float hp, float hop) {
  const float d = x - t, ad = __builtin_fabsf(d);
  switch (kind) {
    case 1: return d * d;
    case 2: return ad;
    case 3: return ad < p ? d * d * hop : ad - hp;
    default: return ad <= p ? 0.5f * d * d : p * (ad - hp);
  }
}
struct RegLossF32 {
  using Out = float; using In0 = float; using In1 = float; using In2 = void;
  static constexpr int NIN = 2;
  int kind;
  float p, hp, hop;
  __device__ __forceinline__ float operator()(float x, float t) const { return regression_term(kind, x, t, p, hp, hop); }
};
struct RegLossDyn {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = Dyn<float>; using In2 = void;
  static constexpr int NIN = 2;
  int kind;
  float p, hp, hop;
  __device__ __forceinline__ float operator()(float x, float t) const { return regression_term(kind, x, t, p, hp, hop); }
};

tx_status regression_elementwise(int kind, double param, const tx_tensor* out, const tx_tensor* x, const tx_tensor* t, hipStream_t s) {
  const tx_tensor* ops[3] = {out, x, t};
  Iter it;
  iter_build(&it, out->ndim, out->sizes, ops, 3);
  const float p = (float)param, hp = (float)(0.5 * param), hop = (float)(0.5 / param);
  if (x->dtype == TX_F32) return launch_ew(it, RegLossF32{kind, p, hp, hop}, s);
  return launch_ew(it, RegLossDyn{kind, p, hp, hop}, s);
}

tx_status regression_checks(int kind, const tx_tensor* out, const tx_tensor* x, const tx_tensor* t, int reduction, double param,
                            int* nd, int64_t* shape) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "input")) || (rc = check_tensor(t, "target"))) return rc;
  if (kind < TX_LOSS_MSE || kind > TX_LOSS_HUBER) return fail(TX_ERR_SCALAR, "loss: unknown kind %d", kind);
  if (!dtype_is_float(x->dtype)) return fail(TX_ERR_DTYPE, "loss: floating dtypes only");
  if (t->dtype != x->dtype || out->dtype != x->dtype) return fail(TX_ERR_DTYPE, "loss: target and out must have input's dtype");
  if (reduction < TX_REDUCTION_NONE || reduction > TX_REDUCTION_SUM) return fail(TX_ERR_SCALAR, "loss: unknown reduction %d", reduction);
  if (kind == TX_LOSS_SMOOTH_L1 && !(param >= 0.0)) return fail(TX_ERR_SCALAR, "smooth_l1_loss: beta must not be negative");
  if (kind == TX_LOSS_HUBER && !(param > 0.0)) return fail(TX_ERR_SCALAR, "huber_loss: delta must be positive");
  const tx_tensor* ins[2] = {x, t};
  if ((rc = broadcast_shapes(ins, 2, nd, shape))) return rc;
  if (reduction == TX_REDUCTION_NONE) {
    if (!same_sizes(out, *nd, shape)) return fail(TX_ERR_SHAPE, "loss: out must have the broadcast shape of input and target");
    return check_out_overlap(out, ins, 2);
  }
  if (out->ndim != 0) return fail(TX_ERR_SHAPE, "loss: a reduced result is 0-dim");
  return TX_OK;
}

constexpr size_t kAlign = 256;
size_t round_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

tx_status bce_checks(const tx_tensor* out, const tx_tensor* x, const tx_tensor* t, const tx_tensor* w, int reduction) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "input")) || (rc = check_tensor(t, "target"))) return rc;
  if (w && (rc = check_tensor(w, "weight"))) return rc;
  if (!dtype_is_float(x->dtype)) return fail(TX_ERR_DTYPE, "binary_cross_entropy takes floating dtypes only");
  if (t->dtype != x->dtype || out->dtype != x->dtype)
    return fail(TX_ERR_DTYPE, "binary_cross_entropy: target and out must have input's dtype");
  if (w && !dtype_is_float(w->dtype)) return fail(TX_ERR_DTYPE, "binary_cross_entropy: weight must be floating");
  if (reduction < TX_REDUCTION_NONE || reduction > TX_REDUCTION_SUM)
    return fail(TX_ERR_SCALAR, "binary_cross_entropy: unknown reduction %d", reduction);
  if (!same_sizes(t, x->ndim, x->sizes)) return fail(TX_ERR_SHAPE, "binary_cross_entropy: target must have input's shape");
  if (w) {
    const tx_tensor* ins[2] = {x, w};
    int nd;
    int64_t shape[TX_MAX_DIMS];
    if ((rc = broadcast_shapes(ins, 2, &nd, shape))) return rc;
    if (!same_sizes(x, nd, shape)) return fail(TX_ERR_SHAPE, "binary_cross_entropy: weight does not broadcast to input's shape");
  }
  if (reduction == TX_REDUCTION_NONE) {
    if (!same_sizes(out, x->ndim, x->sizes)) return fail(TX_ERR_SHAPE, "binary_cross_entropy: out must have input's shape");
    const tx_tensor* ins[3] = {x, t, w};
    return check_out_overlap(out, ins, w ? 3 : 2);
  }
  if (out->ndim != 0) return fail(TX_ERR_SHAPE, "binary_cross_entropy: a reduced result is 0-dim");
  return TX_OK;
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

size_t tx_binary_cross_entropy_workspace_bytes(const tx_tensor* out, const tx_tensor* input, const tx_tensor* target,
                                               const tx_tensor* weight, int reduction) {
  if (bce_checks(out, input, target, weight, reduction) || reduction == TX_REDUCTION_NONE) return 0;
  const int64_t n = numel(input);
  const int es = dtype_size(input->dtype);
  // at most 2048 workgroups write one binary64 partial each
  const size_t partials = round_up((size_t)2048 * sizeof(double));
  if (strcmp(forced_path(), "bce-two-pass") && bce_fused_mode(input, target, weight) >= 0) return partials;
  return partials + round_up((size_t)n * es);
}

tx_status tx_binary_cross_entropy(const tx_tensor* out, const tx_tensor* input, const tx_tensor* target,
                                  const tx_tensor* weight, int reduction, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  tx_status rc = bce_checks(out, input, target, weight, reduction);
  if (rc) return rc;
  set_path("");
  hipStream_t s = as_stream(stream);
  const int64_t n = numel(input);
  if (reduction == TX_REDUCTION_NONE) {
    if (n == 0) return TX_OK;
    return bce_elementwise(out, input, target, weight, s);
  }
  const size_t need = tx_binary_cross_entropy_workspace_bytes(out, input, target, weight, reduction);
  if (!workspace || workspace_bytes < need || (uintptr_t)workspace % 16 != 0)
    return fail(TX_ERR_WORKSPACE, "binary_cross_entropy: workspace of %zu bytes (16-byte aligned) required, got %zu", need,
                workspace_bytes);
  const int mean = reduction == TX_REDUCTION_MEAN;
  const int es = dtype_size(input->dtype);
  double* partial = (double*)workspace;
  const int mode = strcmp(forced_path(), "bce-two-pass") ? bce_fused_mode(input, target, weight) : -1;
  if (mode >= 0 || n == 0) {
    const int64_t last = input->ndim ? input->sizes[input->ndim - 1] : 1;
    return bce_reduce(out, input->dtype, input->data, target->data, weight, mode < 0 ? 0 : mode, n, last, mean, partial, s);
  }
  if (workspace_bytes < round_up((size_t)2048 * sizeof(double)) + round_up((size_t)n * es))
    return fail(TX_ERR_WORKSPACE, "binary_cross_entropy: workspace too small for the two-pass form");
  // losses into the workspace (contiguous, input's dtype), then their sum
  tx_tensor tmp;
  tmp.data = (char*)workspace + round_up((size_t)2048 * sizeof(double));
  tmp.dtype = input->dtype;
  tmp.ndim = input->ndim;
  int64_t stride = 1;
  for (int d = input->ndim - 1; d >= 0; --d) {
    tmp.sizes[d] = input->sizes[d];
    tmp.strides[d] = stride;
    stride *= input->sizes[d];
  }
  if ((rc = bce_elementwise(&tmp, input, target, weight, s))) return rc;
  rc = bce_reduce(out, input->dtype, tmp.data, nullptr, nullptr, 3, n, 1, mean, partial, s);
  set_path("bce-two-pass");
  return rc;
}

size_t tx_loss_workspace_bytes(int kind, const tx_tensor* out, const tx_tensor* input, const tx_tensor* target, int reduction,
                               double param) {
  int nd;
  int64_t shape[TX_MAX_DIMS];
  if (regression_checks(kind, out, input, target, reduction, param, &nd, shape) || reduction == TX_REDUCTION_NONE) return 0;
  const size_t partials = round_up((size_t)2048 * sizeof(double));
  const bool same = same_sizes(target, input->ndim, input->sizes);
  if (same && strcmp(forced_path(), "loss-two-pass") && bce_fused_mode(input, target, nullptr) >= 0) return partials;
  int64_t n = 1;
  for (int d = 0; d < nd; ++d) n *= shape[d];
  return partials + round_up((size_t)n * dtype_size(input->dtype));
}

tx_status tx_loss(int kind, const tx_tensor* out, const tx_tensor* input, const tx_tensor* target, int reduction, double param,
                  void* workspace, size_t workspace_bytes, void* stream) {
  int nd;
  int64_t shape[TX_MAX_DIMS];
  tx_status rc = regression_checks(kind, out, input, target, reduction, param, &nd, shape);
  if (rc) return rc;
  set_path("");
  hipStream_t s = as_stream(stream);
  int64_t n = 1;
  for (int d = 0; d < nd; ++d) n *= shape[d];
  const int k = kind + 1;                               // the kernels' numbering keeps 0 for binary_cross_entropy
  if (reduction == TX_REDUCTION_NONE) {
    if (n == 0) return TX_OK;
    return regression_elementwise(k, param, out, input, target, s);
  }
  const size_t need = tx_loss_workspace_bytes(kind, out, input, target, reduction, param);
  if (!workspace || workspace_bytes < need || (uintptr_t)workspace % 16 != 0)
    return fail(TX_ERR_WORKSPACE, "loss: workspace of %zu bytes (16-byte aligned) required, got %zu", need, workspace_bytes);
  const int mean = reduction == TX_REDUCTION_MEAN;
  double* partial = (double*)workspace;
  const bool same = same_sizes(target, input->ndim, input->sizes);
  const bool fused = same && strcmp(forced_path(), "loss-two-pass") && bce_fused_mode(input, target, nullptr) >= 0;
  if (fused || n == 0)
    return bce_reduce(out, input->dtype, input->data, target->data, nullptr, 0, n, 1, mean, partial, s, k, param);
  // terms into the workspace (contiguous, broadcast shape, input's dtype), then their sum
  tx_tensor tmp;
  tmp.data = (char*)workspace + round_up((size_t)2048 * sizeof(double));
  tmp.dtype = input->dtype;
  tmp.ndim = nd;
  int64_t stride = 1;
  for (int d = nd - 1; d >= 0; --d) {
    tmp.sizes[d] = shape[d];
    tmp.strides[d] = stride;
    stride *= shape[d];
  }
  if ((rc = regression_elementwise(k, param, &tmp, input, target, s))) return rc;
  rc = bce_reduce(out, input->dtype, tmp.data, nullptr, nullptr, 3, n, 1, mean, partial, s);
  set_path("loss-two-pass");
  return rc;
}

}  // extern "C"
