// tx_reduce: validation, planning and dispatch; instantiates the sum / mean /
// var policies (reduce_b.hip holds prod / amax / argmax).
#include <mutex>

#include "reduce_impl.h"

namespace tx {
namespace red {

tx_status normalise_dims(int nd, const int64_t* dims, int ndims, bool* reduced) {
  for (int d = 0; d < TX_MAX_DIMS; ++d) reduced[d] = false;
  if (ndims == 0 || dims == nullptr) {
    for (int d = 0; d < nd; ++d) reduced[d] = true;
    return TX_OK;
  }
  bool seen[TX_MAX_DIMS] = {false};
  for (int i = 0; i < ndims; ++i) {
    int d;
    tx_status rc = wrap_dim(dims[i], nd, &d);
    if (rc) return rc;
    if (seen[d]) return fail(TX_ERR_DIM, "dim %d appears twice", d);
    seen[d] = true;
    if (nd > 0) reduced[d] = true;
  }
  return TX_OK;
}

void plan_dims(Plan* p, const tx_tensor* x, const tx_tensor* out, const bool* reduced, int keepdim) {
  p->nk = p->nr = 0;
  p->nout = p->nred = 1;
  int nred_dims = 0;
  int od = 0;   // running output dim
  for (int d = 0; d < x->ndim; ++d) {
    const int64_t sz = x->sizes[d], xs = x->strides[d];
    if (reduced[d]) {
      ++nred_dims;
      p->nred *= sz;
      if (keepdim) ++od;
      if (sz == 1) continue;
      if (p->nr > 0 && p->rxs[p->nr - 1] == xs * sz) {          // merge into the previous (outer) reduced dim
        p->rsize[p->nr - 1] *= sz;
        p->rxs[p->nr - 1] = xs;
      } else {
        p->rsize[p->nr] = sz;
        p->rxs[p->nr] = xs;
        ++p->nr;
      }
    } else {
      const int64_t os = out->strides[od];
      ++od;
      p->nout *= sz;
      if (sz == 1) continue;
      if (p->nk > 0 && p->kxs[p->nk - 1] == xs * sz && p->kos[p->nk - 1] == os * sz) {
        p->ksize[p->nk - 1] *= sz;
        p->kxs[p->nk - 1] = xs;
        p->kos[p->nk - 1] = os;
      } else {
        p->ksize[p->nk] = sz;
        p->kxs[p->nk] = xs;
        p->kos[p->nk] = os;
        ++p->nk;
      }
    }
  }
  p->single_dim = nred_dims == 1;
  if (p->nr == 0) { p->nr = 1; p->rsize[0] = 1; p->rxs[0] = 0; }
}

static bool multiple_of(int64_t v, int64_t m) { return v % m == 0; }

void plan_launch(Plan* p, const tx_tensor* x, int esize, bool) {
  const int V = 16 / esize;
  const bool red_contig = p->rxs[p->nr - 1] == 1 && p->rsize[p->nr - 1] > 1;
  const bool kept_contig = p->nk > 0 && p->kxs[p->nk - 1] == 1 && p->kos[p->nk - 1] == 1;
  p->kind = (kept_contig && !red_contig && p->ksize[p->nk - 1] >= 16) ? 1 : 0;
  const bool base_al = ((uintptr_t)x->data % 16) == 0;
  p->vec = 1;
  p->nv = 1;
  p->split = 1;
  p->chunk = p->nred;
  if (p->kind == 0) {
    bool ok = red_contig && base_al && multiple_of(p->rsize[p->nr - 1], V);
    for (int d = 0; ok && d < p->nr - 1; ++d) ok = multiple_of(p->rxs[d] * esize, 16);
    for (int d = 0; ok && d < p->nk; ++d) ok = multiple_of(p->kxs[d] * esize, 16);
    if (ok) p->vec = V;
    // a workgroup per output only when the innermost reduced run is long enough for four consecutive
    // 256-lane steps to stay inside it; with a shorter run (say 4 KiB rows of a second reduced dim) the four
    // loads a lane keeps in flight would sit a whole outer stride apart, and a wave per output reads them as
    // one contiguous piece instead
    p->group = (p->rsize[p->nr - 1] * esize >= 16384) ? kBlock : kWave;
    // rows of 1 to 2 KiB, and many of them: half a wave per row, so that a lane still has four vectors in flight and
    // a workgroup covers 8 rows (a wave per 2 KiB row leaves two loads per lane and twice the workgroups)
    if (p->vec > 1 && p->nr == 1 && p->nred * esize > 1024 && p->nred * esize <= 2048 && p->nout >= 65536 &&
        strcmp(forced_path(), "rows-wave") != 0)
      p->group = kWave / 2;
    const int gpb = kBlock / p->group;
    p->blocks_x = (p->nout + gpb - 1) / gpb;
    const int64_t step = (int64_t)p->group * p->vec;
    if (p->blocks_x < 512 && p->nred >= step * 16) {
      int64_t s = std::min<int64_t>(kMaxSplit, (2048 + p->blocks_x - 1) / p->blocks_x);
      s = std::min<int64_t>(s, p->nred / (step * 8));
      if (s > 1) {
        int64_t chunk = (p->nred + s - 1) / s;
        chunk = (chunk + step - 1) / step * step;
        p->chunk = chunk;
        p->split = (int)((p->nred + chunk - 1) / chunk);
      }
    }
  } else {
    bool ok = base_al && multiple_of(p->ksize[p->nk - 1], V);
    for (int d = 0; ok && d < p->nr; ++d) ok = multiple_of(p->rxs[d] * esize, 16);
    for (int d = 0; ok && d < p->nk - 1; ++d) ok = multiple_of(p->kxs[d] * esize, 16);
    if (ok) p->vec = V;
    p->group = 1;
    const int64_t threads = (p->nout + p->vec - 1) / p->vec;
    // four vectors per thread for 4- and 8-byte elements while that still leaves four workgroups per compute
    // unit (sum of fp32 [64,4096,1024] over dim 0: 171 us against 202 us with one); 2-byte elements measured
    // fastest with one vector per thread
    p->nv = (p->vec > 1 && p->nr == 1 && esize >= 4 && threads >= 4 * 1024 * kBlock) ? 4 : 1;
    if (!strcmp(forced_path(), "cols-nv1")) p->nv = 1;
    if (!strcmp(forced_path(), "cols-nv2") && p->vec > 1 && p->nr == 1) p->nv = 2;
    if (!strcmp(forced_path(), "cols-nv4") && p->vec > 1 && p->nr == 1) p->nv = 4;
    p->blocks_x = (threads + kBlock * p->nv - 1) / (kBlock * p->nv);
    if (p->blocks_x < 512 && p->nred >= 64) {
      int64_t s = std::min<int64_t>(kMaxSplit, (1024 + p->blocks_x - 1) / p->blocks_x);
      s = std::min<int64_t>(s, p->nred / 16);
      if (s > 1) {
        p->chunk = (p->nred + s - 1) / s;
        p->split = (int)((p->nred + p->chunk - 1) / p->chunk);
      }
    }
  }
}

size_t plan_ws_bytes(const Plan& p, size_t acc) { return p.split > 1 ? (size_t)p.nout * p.split * acc : 0; }

size_t acc_size(int op, int dtype) {
  const bool flt = dtype_is_float(dtype);
  switch (op) {
    case TX_SUM: case TX_MEAN: return flt ? 4 : 8;
    case TX_PROD: return 8;
    case TX_AMAX: return flt ? 4 : 8;
    case TX_ARGMAX: case TX_ARGMIN: return 16;
    case TX_VAR: case TX_STD: return 16;
    case TX_AMIN: return flt ? 4 : 8;
    case TX_ANY: case TX_ALL: return 8;
    case TX_LOGSUMEXP: return 8;
    case TX_NANSUM: return flt ? 16 : 8;
    case TX_NANMEAN: return 16;
    case TX_COUNT_NONZERO: case TX_NORM: return 8;
  }
  return 16;
}

#define TX_DISPATCH_DTYPE(POLICY, ...)                                                               \
  switch (x->dtype) {                                                                                \
    case TX_F32: return launch<POLICY<float __VA_ARGS__>>(p, x, out, c, ws, wsb, s);                  \
    case TX_BF16: return launch<POLICY<bf16 __VA_ARGS__>>(p, x, out, c, ws, wsb, s);                  \
    case TX_F16: return launch<POLICY<f16 __VA_ARGS__>>(p, x, out, c, ws, wsb, s);                    \
    default: break;                                                                                  \
  }

tx_status launch_sum(bool mean, const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                     hipStream_t s) {
  if (mean) {
#define COMMA_TRUE , true
    TX_DISPATCH_DTYPE(SumPolicy, COMMA_TRUE)
    return fail(TX_ERR_DTYPE, "mean takes floating dtypes only");
  }
#define COMMA_FALSE , false
  TX_DISPATCH_DTYPE(SumPolicy, COMMA_FALSE)
  switch (x->dtype) {
    case TX_I64: return launch<SumPolicy<int64_t, false>>(p, x, out, c, ws, wsb, s);
    case TX_I32: return launch<SumPolicy<int32_t, false>>(p, x, out, c, ws, wsb, s);
    default: return launch<SumPolicy<uint8_t, false>>(p, x, out, c, ws, wsb, s);
  }
}

tx_status launch_var(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                     hipStream_t s) {
  TX_DISPATCH_DTYPE(VarPolicy)
  return fail(TX_ERR_DTYPE, "var takes floating dtypes only");
}

tx_status build_plan(int op, const tx_tensor* x, const tx_tensor* out, const int64_t* dims, int32_t ndims, int keepdim,
                     Plan* p) {
  bool reduced[TX_MAX_DIMS];
  tx_status rc = normalise_dims(x->ndim, dims, ndims, reduced);
  if (rc) return rc;
  plan_dims(p, x, out, reduced, keepdim);
  if ((p->nk > 1 && p->nout >= (1ll << 31)) || (p->nr > 1 && p->nred >= (1ll << 31)))
    return fail(TX_ERR_UNSUPPORTED, "reduction extents beyond 2^31 with non-mergeable dims");
  plan_launch(p, x, dtype_size(x->dtype), op == TX_VAR || op == TX_STD);
  p->aux = (op == TX_STD || op == TX_ALL) ? 1.0 : 0.0;
  if (p->blocks_x >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "too many outputs for one launch");
  return TX_OK;
}

}  // namespace red
}  // namespace tx

using namespace tx;
using namespace tx::red;

static tx_status reduce_checks(int op, const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims,
                               int keepdim) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x"))) return rc;
  int32_t rd, nd;
  int64_t shape[TX_MAX_DIMS];
  if ((rc = tx_infer_reduce(op, x, dims, ndims, keepdim, &rd, &nd, shape))) return rc;
  const bool widen = dtype_is_float(rd) && out->dtype == TX_F32 && op != TX_AMAX && op != TX_AMIN;
  if (out->dtype != rd && !widen)
    return fail(TX_ERR_DTYPE, "out dtype %s, expected %s", dtype_name(out->dtype), dtype_name(rd));
  if (!same_sizes(out, nd, shape)) return fail(TX_ERR_SHAPE, "out does not have the reduced shape");
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  if (partial_overlap(out, x) || (out->data == x->data && numel(out) && numel(x)))
    return fail(TX_ERR_OVERLAP, "out overlaps the input");
  return TX_OK;
}

namespace {

// Scratch of the entry point that allocates nothing: one array per GPU, held until the process ends.  The name is a
// host-side stand-in; the device address comes from hipGetSymbolAddress, once per device, and only that address is
// handed to kernels.
constexpr size_t kStaticScratchBytes = TX_REDUCE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

tx_status static_scratch(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(TX_ERR_LAUNCH, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(TX_ERR_LAUNCH, "device ordinal %d is outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(TX_ERR_LAUNCH, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return TX_OK;
}

tx_status reduce_dispatch(int op, const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims, int keepdim,
                          double correction, void* ws, size_t ws_bytes, void* stream) {
  tx_status rc = reduce_checks(op, out, x, dims, ndims, keepdim);
  if (rc) return rc;
  set_path("");
  Plan p;
  if ((rc = build_plan(op, x, out, dims, ndims, keepdim, &p))) return rc;
  if (p.nout == 0) return TX_OK;
  if ((op == TX_AMAX || op == TX_ARGMAX || op == TX_AMIN || op == TX_ARGMIN) && p.nred == 0)
    return fail(TX_ERR_EMPTY_REDUCTION, "amax / amin / argmax / argmin over an empty extent");
  if (op == TX_NORM) {                                   // correction carries the exponent p
    if (correction != correction) return fail(TX_ERR_SCALAR, "norm: the exponent is NaN");
    if (p.nred == 0 && (correction < 0.0 || correction == __builtin_inf()))
      return fail(TX_ERR_EMPTY_REDUCTION, "norm with an infinite or negative exponent over an empty extent");
  }
  hipStream_t s = as_stream(stream);
  switch (op) {
    case TX_NANSUM: return launch_nansum(false, p, x, out, correction, ws, ws_bytes, s);
    case TX_NANMEAN: return launch_nansum(true, p, x, out, correction, ws, ws_bytes, s);
    case TX_COUNT_NONZERO: return launch_count(p, x, out, correction, ws, ws_bytes, s);
    case TX_NORM: return launch_norm(p, x, out, correction, ws, ws_bytes, s);
    case TX_SUM: return launch_sum(false, p, x, out, correction, ws, ws_bytes, s);
    case TX_MEAN: return launch_sum(true, p, x, out, correction, ws, ws_bytes, s);
    case TX_VAR: return launch_var(p, x, out, correction, ws, ws_bytes, s);
    case TX_PROD: return launch_prod(p, x, out, correction, ws, ws_bytes, s);
    case TX_AMAX: return launch_amax(p, x, out, correction, ws, ws_bytes, s);
    case TX_ARGMAX: return launch_argmax(p, x, out, correction, ws, ws_bytes, s);
    case TX_STD: return launch_var(p, x, out, correction, ws, ws_bytes, s);          // Plan::aux asks for the square root
    case TX_AMIN: return launch_amin(p, x, out, correction, ws, ws_bytes, s);
    case TX_ARGMIN: return launch_argmin(p, x, out, correction, ws, ws_bytes, s);
    case TX_ANY: case TX_ALL: return launch_anyall(p, x, out, correction, ws, ws_bytes, s);
    case TX_LOGSUMEXP: return launch_logsumexp(p, x, out, correction, ws, ws_bytes, s);
  }
  return fail(TX_ERR_DTYPE, "unknown reduce op %d", op);
}

}  // namespace

extern "C" {

tx_status tx_infer_reduce(int op, const tx_tensor* x, const int64_t* dims, int32_t ndims, int keepdim, int32_t* dtype,
                          int32_t* ndim, int64_t* sizes) {
  if (!x) return fail(TX_ERR_NULL, "infer_reduce: null descriptor");
  if (x->ndim < 0 || x->ndim > TX_MAX_DIMS) return fail(TX_ERR_NDIM, "infer_reduce: bad ndim");
  if (!dtype_valid(x->dtype)) return fail(TX_ERR_DTYPE, "infer_reduce: bad dtype code");
  const bool flt = dtype_is_float(x->dtype);
  int rd;
  switch (op) {
    case TX_SUM: case TX_PROD: rd = flt ? x->dtype : TX_I64; break;
    case TX_MEAN: case TX_VAR: case TX_STD:
      if (!flt) return fail(TX_ERR_DTYPE, "mean / var / std take floating dtypes only");
      rd = x->dtype;
      break;
    case TX_LOGSUMEXP: rd = flt ? x->dtype : TX_F32; break;     // bool / integer input is converted to fp32
    case TX_AMAX: case TX_AMIN: rd = x->dtype; break;
    case TX_ARGMAX: case TX_ARGMIN:
      if (x->dtype == TX_BOOL) return fail(TX_ERR_DTYPE, "argmax / argmin do not take bool");
      rd = TX_I64;
      break;
    case TX_ANY: case TX_ALL: rd = TX_BOOL; break;
    case TX_NANSUM: rd = flt ? x->dtype : TX_I64; break;
    case TX_NANMEAN: case TX_NORM:
      if (!flt) return fail(TX_ERR_DTYPE, "nanmean / norm take floating dtypes only");
      rd = x->dtype;
      break;
    case TX_COUNT_NONZERO: rd = TX_I64; break;
    default: return fail(TX_ERR_DTYPE, "unknown reduce op %d", op);
  }
  if ((op == TX_PROD || op == TX_ARGMAX || op == TX_ARGMIN) && ndims > 1 && dims)
    return fail(TX_ERR_DIM, "prod / argmax / argmin reduce one dim or all dims");
  bool reduced[TX_MAX_DIMS];
  tx_status rc = normalise_dims(x->ndim, dims, ndims, reduced);
  if (rc) return rc;
  int nd = 0;
  for (int d = 0; d < x->ndim; ++d) {
    if (reduced[d]) { if (keepdim) { if (sizes) sizes[nd] = 1; ++nd; } }
    else { if (sizes) sizes[nd] = x->sizes[d]; ++nd; }
  }
  if (dtype) *dtype = rd;
  if (ndim) *ndim = nd;
  return TX_OK;
}

tx_status tx_reduce(int op, const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims, int keepdim,
                    double correction, void* ws, size_t ws_bytes, void* stream) {
  return reduce_dispatch(op, out, x, dims, ndims, keepdim, correction, ws, ws_bytes, stream);
}

tx_status tx_reduce_static(int op, const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims,
                           int keepdim, double correction, void* stream) {
  tx_status rc = reduce_checks(op, out, x, dims, ndims, keepdim);
  if (rc) return rc;
  Plan p;
  if ((rc = build_plan(op, x, out, dims, ndims, keepdim, &p))) return rc;
  const size_t need = plan_ws_bytes(p, acc_size(op, x->dtype));
  if (need > kStaticScratchBytes)
    return fail(TX_ERR_WORKSPACE, "tx_reduce_static: this reduction needs %zu bytes of scratch, the built-in buffer holds %zu; "
                                  "use tx_reduce with a caller workspace", need, kStaticScratchBytes);
  void* ws = nullptr;
  if (need > 0 && (rc = static_scratch(&ws))) return rc;
  return reduce_dispatch(op, out, x, dims, ndims, keepdim, correction, ws, kStaticScratchBytes, stream);
}

size_t tx_reduce_workspace_bytes(int op, const tx_tensor* out, const tx_tensor* x, const int64_t* dims, int32_t ndims,
                                 int keepdim) {
  if (reduce_checks(op, out, x, dims, ndims, keepdim)) return 0;
  Plan p;
  if (build_plan(op, x, out, dims, ndims, keepdim, &p)) return 0;
  return plan_ws_bytes(p, acc_size(op, x->dtype));
}

}  // extern "C"
