// cumprod and logcumsumexp: the scan kernels of scan_impl.h with a product or a log-add-exp as the combining
// operation.  A contiguous operated dim takes the look-back / row-carry kernels; any other layout takes the
// one-lane-per-slice kernel.
#include "scan_impl.h"

namespace tx {
namespace {

tx_status scan_dispatch(int op, const tx_tensor* out, const tx_tensor* x, int dim, void* ws, size_t wsb, hipStream_t s,
                        size_t* query) {
  const bool wide = out->dtype == TX_F32;
  if (op == TX_SCAN_PROD) {
    // floats multiply in binary64: a product of n factors in fp32 drifts by up to n half-ulps
    switch (x->dtype) {
      case TX_BOOL: return cumsum_launch<uint8_t, int64_t, int64_t, ScanMul>(out, x, dim, ws, wsb, s, query);
      case TX_I32: return cumsum_launch<int32_t, int64_t, int64_t, ScanMul>(out, x, dim, ws, wsb, s, query);
      case TX_I64: return cumsum_launch<int64_t, int64_t, int64_t, ScanMul>(out, x, dim, ws, wsb, s, query);
      case TX_F32: return cumsum_launch<float, float, double, ScanMul>(out, x, dim, ws, wsb, s, query);
      case TX_BF16:
        return wide ? cumsum_launch<bf16, float, double, ScanMul>(out, x, dim, ws, wsb, s, query)
                    : cumsum_launch<bf16, bf16, double, ScanMul>(out, x, dim, ws, wsb, s, query);
      default:
        return wide ? cumsum_launch<f16, float, double, ScanMul>(out, x, dim, ws, wsb, s, query)
                    : cumsum_launch<f16, f16, double, ScanMul>(out, x, dim, ws, wsb, s, query);
    }
  }
  switch (x->dtype) {
    case TX_F32: return cumsum_launch<float, float, LsePair, ScanLse>(out, x, dim, ws, wsb, s, query);
    case TX_BF16:
      return wide ? cumsum_launch<bf16, float, LsePair, ScanLse>(out, x, dim, ws, wsb, s, query)
                  : cumsum_launch<bf16, bf16, LsePair, ScanLse>(out, x, dim, ws, wsb, s, query);
    default:
      return wide ? cumsum_launch<f16, float, LsePair, ScanLse>(out, x, dim, ws, wsb, s, query)
                  : cumsum_launch<f16, f16, LsePair, ScanLse>(out, x, dim, ws, wsb, s, query);
  }
}

tx_status scan_checks(int op, const tx_tensor* out, const tx_tensor* x, int64_t dim, int* d) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x"))) return rc;
  if (op != TX_SCAN_PROD && op != TX_SCAN_LOGSUMEXP) return fail(TX_ERR_SCALAR, "scan: unknown operation %d", op);
  const bool flt = dtype_is_float(x->dtype);
  if (op == TX_SCAN_LOGSUMEXP && !flt) return fail(TX_ERR_DTYPE, "logcumsumexp takes floating dtypes only");
  if (flt) {
    if (out->dtype != x->dtype && out->dtype != TX_F32) return fail(TX_ERR_DTYPE, "scan: out dtype");
  } else if (out->dtype != TX_I64) {
    return fail(TX_ERR_DTYPE, "cumprod of bool / integer input returns int64");
  }
  if (!same_sizes(out, x->ndim, x->sizes)) return fail(TX_ERR_SHAPE, "scan: out must have x's shape");
  if ((rc = wrap_dim(dim, x->ndim, d))) return rc;
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  if (partial_overlap(out, x) || (out->data == x->data && numel(x) > 0)) return fail(TX_ERR_OVERLAP, "scan: out must not alias x");
  return TX_OK;
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

tx_status tx_scan(int op, const tx_tensor* out, const tx_tensor* x, int64_t dim, void* ws, size_t ws_bytes, void* stream) {
  if (op == TX_SCAN_SUM) return tx_cumsum(out, x, dim, ws, ws_bytes, stream);
  int d;
  tx_status rc = scan_checks(op, out, x, dim, &d);
  if (rc) return rc;
  set_path("");
  if (numel(x) == 0) return TX_OK;
  return scan_dispatch(op, out, x, d, ws, ws_bytes, as_stream(stream), nullptr);
}

size_t tx_scan_workspace_bytes(int op, const tx_tensor* out, const tx_tensor* x, int64_t dim) {
  if (op == TX_SCAN_SUM) return tx_cumsum_workspace_bytes(out, x, dim);
  int d;
  if (scan_checks(op, out, x, dim, &d)) return 0;
  if (numel(x) == 0) return 0;
  size_t q = 0;
  scan_dispatch(op, out, x, d, nullptr, 0, nullptr, &q);
  return q;
}

}  // extern "C"
