// Data-moving shape operators: copy with dtype conversion (clone, contiguous, to, expand made real, copy_) on the
// elementwise iterator, and flip / roll / tril / triu as one index-remapping copy kernel that moves raw bits.
#include "ew_impl.h"
#include "index_util.h"

namespace tx {
namespace {

// ---------------------------------------------------------------------------
// copy with conversion
// ---------------------------------------------------------------------------
template <class B> struct CopyBits {
  using Out = B; using In0 = B; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ B operator()(B v) const { return v; }
};
template <class To, class From> struct CastTyped {                  // fp32 <-> half types: one conversion instruction
  using Out = To; using In0 = From; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ To operator()(From v) const { return cvt<To>(cvt<float>(v)); }
};
// any source into a floating destination: a floating value is rounded once by the store, an integer goes
// through fp32 (the load's conversion)
struct CastToFloat {
  using Out = Dyn<float>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  __device__ __forceinline__ float operator()(float v) const { return v; }
};
// floating source into an integer (truncated toward zero) or bool (not zero) destination
struct CastFloatToInt {
  using Out = Dyn<int64_t>; using In0 = Dyn<float>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int to_bool;
  __device__ __forceinline__ int64_t operator()(float v) const { return to_bool ? (int64_t)(v != 0.0f) : (int64_t)v; }
};
struct CastIntToInt {                                                // the store wraps to int32; a bool target gets 0 / 1
  using Out = Dyn<int64_t>; using In0 = Dyn<int64_t>; using In1 = void; using In2 = void;
  static constexpr int NIN = 1;
  int to_bool;
  __device__ __forceinline__ int64_t operator()(int64_t v) const { return to_bool ? (int64_t)(v != 0) : v; }
};

// ---------------------------------------------------------------------------
// flip / roll / tril / triu: out[idx] = x[map(idx)] or 0
// ---------------------------------------------------------------------------
struct RemapArgs {
  const char* x;
  char* out;
  Dims shape;                       // out's shape, innermost dim counted in vectors
  int64_t xs[TX_MAX_DIMS], os[TX_MAX_DIMS];     // strides in elements (innermost: in vectors' first elements)
  int mode[TX_MAX_DIMS];            // 0 same coordinate, 1 flipped, 2 rolled by shift
  int64_t shift[TX_MAX_DIMS], size[TX_MAX_DIMS];
  int tri;                          // 0 none, 1 tril, 2 triu
  int64_t diagonal;
};

// One lane per VEC consecutive elements of the innermost dim (VEC > 1 only when that dim keeps its coordinate or is
// flipped, and is contiguous on both sides).  B: an unsigned integer of the element's size.
template <class B, int VEC>
__global__ __launch_bounds__(kBlock) void remap_copy_kernel(const RemapArgs a) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t >= a.shape.numel) return;
  uint32_t rem = (uint32_t)t;
  int64_t xo = 0, oo = 0, ci = 0, cj = 0;
  const int nd = a.shape.n;
  for (int d = nd - 1; d >= 0; --d) {
    uint32_t q, c;
    a.shape.div[d].divmod(rem, q, c);
    rem = q;
    int64_t o = c, sidx = c;
    if (d == nd - 1) { o *= VEC; sidx = o; cj = o; }
    if (d == nd - 2) ci = c;
    if (a.mode[d] == 1) sidx = a.size[d] - (d == nd - 1 ? VEC : 1) - sidx;      // innermost: the mirrored vector, reversed below
    else if (a.mode[d] == 2) { sidx -= a.shift[d]; if (sidx < 0) sidx += a.size[d]; }
    xo += sidx * a.xs[d];
    oo += o * a.os[d];
  }
  Vec<B, VEC> v = vec_load<B, VEC, true>((const B*)a.x + xo);
  if (VEC > 1 && nd > 0 && a.mode[nd - 1] == 1) {
    Vec<B, VEC> r;
#pragma unroll
    for (int e = 0; e < VEC; ++e) r.v[e] = v.v[VEC - 1 - e];
    v = r;
  }
  if (a.tri) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const int64_t off = cj + e - ci;
      const bool keep = a.tri == 2 ? off >= a.diagonal : off <= a.diagonal;
      if (!keep) v.v[e] = B(0);
    }
  }
  vec_store<B, VEC, true>((B*)a.out + oo, v);
}

template <class B>
tx_status remap_launch(RemapArgs& a, const tx_tensor* out, const tx_tensor* x, bool inner_moves, hipStream_t s) {
  constexpr int V = 16 / (int)sizeof(B);
  const int nd = x->ndim;
  int64_t sizes[TX_MAX_DIMS];
  for (int d = 0; d < nd; ++d) sizes[d] = x->sizes[d];
  bool vec = nd >= 1 && !inner_moves && x->strides[nd - 1] == 1 && out->strides[nd - 1] == 1 && x->sizes[nd - 1] % V == 0 &&
             (uintptr_t)x->data % 16 == 0 && (uintptr_t)out->data % 16 == 0;
  for (int d = 0; vec && d < nd - 1; ++d) vec = x->strides[d] % V == 0 && out->strides[d] % V == 0;
  if (vec) sizes[nd - 1] /= V;
  fill_dims(&a.shape, nd, sizes);
  if (a.shape.numel >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "more than 2^31 elements (or vectors) to move");
  const unsigned grid = (unsigned)((a.shape.numel + kBlock - 1) / kBlock);
  set_path(vec ? "remap-vec" : "remap");
  if (vec) hipLaunchKernelGGL((remap_copy_kernel<B, V>), dim3(grid), dim3(kBlock), 0, s, a);
  else hipLaunchKernelGGL((remap_copy_kernel<B, 1>), dim3(grid), dim3(kBlock), 0, s, a);
  return check_launch("index-remapping copy kernel");
}

tx_status remap_dispatch(RemapArgs& a, const tx_tensor* out, const tx_tensor* x, bool inner_moves, hipStream_t s) {
  a.x = (const char*)x->data;
  a.out = (char*)out->data;
  for (int d = 0; d < x->ndim; ++d) {
    a.xs[d] = x->strides[d];
    a.os[d] = out->strides[d];
    a.size[d] = x->sizes[d];
  }
  switch (dtype_size(x->dtype)) {
    case 1: return remap_launch<uint8_t>(a, out, x, inner_moves, s);
    case 2: return remap_launch<uint16_t>(a, out, x, inner_moves, s);
    case 4: return remap_launch<uint32_t>(a, out, x, inner_moves, s);
    default: return remap_launch<uint64_t>(a, out, x, inner_moves, s);
  }
}

tx_status remap_checks(const char* name, const tx_tensor* out, const tx_tensor* x) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x"))) return rc;
  if (out->dtype != x->dtype) return fail(TX_ERR_DTYPE, "%s: out must have x's dtype", name);
  if (!same_sizes(out, x->ndim, x->sizes)) return fail(TX_ERR_SHAPE, "%s: out must have x's shape", name);
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  if (partial_overlap(out, x) || (out->data == x->data && numel(x) > 0)) return fail(TX_ERR_OVERLAP, "%s: out must not alias x", name);
  return TX_OK;
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

tx_status tx_copy(const tx_tensor* out, const tx_tensor* x, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x"))) return rc;
  const tx_tensor* both[2] = {out, x};
  int nd;
  int64_t shape[TX_MAX_DIMS];
  if ((rc = broadcast_shapes(both, 2, &nd, shape))) return rc;
  if (!same_sizes(out, nd, shape)) return fail(TX_ERR_SHAPE, "copy: x does not broadcast to out's shape");
  const tx_tensor* ins[1] = {x};
  if ((rc = check_out_overlap(out, ins, 1))) return rc;
  set_path("");
  if (numel(out) == 0) return TX_OK;
  Iter it;
  iter_build(&it, nd, shape, both, 2);
  hipStream_t s = as_stream(stream);
  const int from = x->dtype, to = out->dtype;
  if (from == to) {
    switch (dtype_size(to)) {
      case 1: return launch_ew(it, CopyBits<uint8_t>{}, s);
      case 2: return launch_ew(it, CopyBits<uint16_t>{}, s);
      case 4: return launch_ew(it, CopyBits<uint32_t>{}, s);
      default: return launch_ew(it, CopyBits<uint64_t>{}, s);
    }
  }
  if (from == TX_F32 && to == TX_BF16) return launch_ew(it, CastTyped<bf16, float>{}, s);
  if (from == TX_F32 && to == TX_F16) return launch_ew(it, CastTyped<f16, float>{}, s);
  if (from == TX_BF16 && to == TX_F32) return launch_ew(it, CastTyped<float, bf16>{}, s);
  if (from == TX_F16 && to == TX_F32) return launch_ew(it, CastTyped<float, f16>{}, s);
  if (dtype_is_float(to)) return launch_ew(it, CastToFloat{}, s);
  if (dtype_is_float(from)) return launch_ew(it, CastFloatToInt{to == TX_BOOL}, s);
  return launch_ew(it, CastIntToInt{to == TX_BOOL}, s);
}

tx_status tx_flip(const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims, void* stream) {
  tx_status rc = remap_checks("flip", out, x);
  if (rc) return rc;
  RemapArgs a;
  memset(&a, 0, sizeof(a));
  for (int i = 0; i < ndims; ++i) {
    int d;
    if ((rc = wrap_dim(dims[i], x->ndim, &d))) return rc;
    if (x->ndim == 0) continue;
    if (a.mode[d]) return fail(TX_ERR_DIM, "flip: dim %d listed twice", d);
    a.mode[d] = 1;
  }
  set_path("");
  if (numel(x) == 0) return TX_OK;
  return remap_dispatch(a, out, x, false, as_stream(stream));      // a flipped innermost dim still moves whole vectors
}

tx_status tx_roll(const tx_tensor* out, const tx_tensor* x, const int64_t* shifts, const int64_t* dims, int32_t n, void* stream) {
  tx_status rc = remap_checks("roll", out, x);
  if (rc) return rc;
  RemapArgs a;
  memset(&a, 0, sizeof(a));
  for (int i = 0; i < n; ++i) {
    int d;
    if ((rc = wrap_dim(dims[i], x->ndim, &d))) return rc;
    if (x->ndim == 0 || x->sizes[d] == 0) continue;
    const int64_t sz = x->sizes[d];
    a.shift[d] = ((a.shift[d] + shifts[i]) % sz + sz) % sz;              // a dim listed twice: the shifts add up
  }
  for (int d = 0; d < x->ndim; ++d) a.mode[d] = a.shift[d] ? 2 : 0;
  set_path("");
  if (numel(x) == 0) return TX_OK;
  return remap_dispatch(a, out, x, x->ndim > 0 && a.mode[x->ndim - 1] != 0, as_stream(stream));
}

tx_status tx_tri(const tx_tensor* out, const tx_tensor* x, int64_t diagonal, int upper, void* stream) {
  tx_status rc = remap_checks(upper ? "triu" : "tril", out, x);
  if (rc) return rc;
  if (x->ndim < 2) return fail(TX_ERR_NDIM, "tril / triu need at least two dims");
  RemapArgs a;
  memset(&a, 0, sizeof(a));
  a.tri = upper ? 2 : 1;
  a.diagonal = diagonal;
  set_path("");
  if (numel(x) == 0) return TX_OK;
  return remap_dispatch(a, out, x, false, as_stream(stream));
}

}  // extern "C"
