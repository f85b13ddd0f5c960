// Host-side operand iterator: turns N broadcast operands into a collapsed,
// output-ordered set of (size, per-operand stride) dims that kernels index.
#pragma once
#include "common.h"

namespace tx {

constexpr int kMaxOperands = 4;

struct IterOperand {
  char* data;
  int dtype;
  int64_t stride[TX_MAX_DIMS];   // elements; dims run outer -> inner
};

struct Iter {
  int ndim;                       // >= 1 (a 0-dim problem becomes one dim of size 1)
  int64_t size[TX_MAX_DIMS];
  int nops;                       // operand 0 is the output
  IterOperand op[kMaxOperands];
  int64_t numel;
};

// `shape` (rank nd) is the broadcast shape and the shape of ops[0]; the other
// operands broadcast against it right-aligned.  Size-1 dims are dropped,
// broadcast dims get stride 0, dims are ordered by decreasing output stride
// and adjacent dims that are jointly contiguous in every operand are merged.
void iter_build(Iter* it, int nd, const int64_t* shape, const tx_tensor* const* ops, int nops);

// Output / aliasing rules shared by the elementwise entry points.
tx_status check_out_overlap(const tx_tensor* out, const tx_tensor* const* ins, int nins);

}  // namespace tx
