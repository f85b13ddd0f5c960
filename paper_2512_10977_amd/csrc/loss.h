// binary_cross_entropy pieces shared between the translation unit that owns the entry point (elementwise form,
// dispatch) and the one that owns the fused reduction kernels.
#pragma once
#include "common.h"

namespace tx {

// how the fused sum / mean kernel can read the operands: -1 = it cannot (the losses are formed first), else the
// weight mode: 0 none, 1 weight laid out like x, 2 one weight per element of the last dim
int bce_fused_mode(const tx_tensor* x, const tx_tensor* t, const tx_tensor* w);
// number of binary64 partials the fused kernel writes for n elements of esize bytes
size_t bce_partial_count(int64_t n, int esize);
// sum (mean != 0: mean) of the losses into the 0-dim `out`.  mode 3: `x` holds n precomputed losses, contiguous
// kind 0: binary_cross_entropy terms; 1 mse, 2 l1, 3 smooth_l1 (param = beta), 4 huber (param = delta): no weight
tx_status bce_reduce(const tx_tensor* out, int dtype, const void* x, const void* t, const tx_tensor* w, int mode, int64_t n,
                     int64_t last, int mean, double* partial, hipStream_t stream, int kind = 0, double param = 1.0);

}  // namespace tx
