#include "iter.h"

#include <algorithm>

namespace tx {

void iter_build(Iter* it, int nd, const int64_t* shape, const tx_tensor* const* ops, int nops) {
  it->nops = nops;
  it->numel = 1;
  for (int d = 0; d < nd; ++d) it->numel *= shape[d];
  for (int o = 0; o < nops; ++o) {
    it->op[o].data = (char*)ops[o]->data;
    it->op[o].dtype = ops[o]->dtype;
  }
  // 1. keep dims of extent != 1, with broadcast strides
  int n = 0;
  int64_t size[TX_MAX_DIMS], stride[kMaxOperands][TX_MAX_DIMS];
  for (int d = 0; d < nd; ++d) {
    if (shape[d] == 1) continue;
    size[n] = shape[d];
    for (int o = 0; o < nops; ++o) {
      int od = d - (nd - ops[o]->ndim);
      stride[o][n] = (od < 0 || ops[o]->sizes[od] == 1) ? 0 : ops[o]->strides[od];
    }
    ++n;
  }
  // 2. order by decreasing output stride (stable insertion sort)
  for (int i = 1; i < n; ++i) {
    for (int j = i; j > 0 && stride[0][j] > stride[0][j - 1]; --j) {
      std::swap(size[j], size[j - 1]);
      for (int o = 0; o < nops; ++o) std::swap(stride[o][j], stride[o][j - 1]);
    }
  }
  // 3. merge dim i into dim i+1 when every operand steps through them as one run
  int m = 0;   // number of merged dims written so far (built from the inner end)
  int64_t msize[TX_MAX_DIMS], mstride[kMaxOperands][TX_MAX_DIMS];
  for (int d = n - 1; d >= 0; --d) {
    bool merge = m > 0;
    if (merge)
      for (int o = 0; o < nops; ++o)
        if (stride[o][d] != mstride[o][m - 1] * msize[m - 1]) { merge = false; break; }
    if (merge) {
      msize[m - 1] *= size[d];
    } else {
      msize[m] = size[d];
      for (int o = 0; o < nops; ++o) mstride[o][m] = stride[o][d];
      ++m;
    }
  }
  if (m == 0) {
    m = 1;
    msize[0] = 1;
    for (int o = 0; o < nops; ++o) mstride[o][0] = 0;
  }
  it->ndim = m;
  for (int d = 0; d < m; ++d) {        // reverse back to outer -> inner
    it->size[d] = msize[m - 1 - d];
    for (int o = 0; o < nops; ++o) it->op[o].stride[d] = mstride[o][m - 1 - d];
  }
}

tx_status check_out_overlap(const tx_tensor* out, const tx_tensor* const* ins, int nins) {
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements (zero or folded strides)");
  for (int i = 0; i < nins; ++i)
    if (partial_overlap(out, ins[i])) return fail(TX_ERR_OVERLAP, "out partially overlaps input %d", i);
  return TX_OK;
}

}  // namespace tx
