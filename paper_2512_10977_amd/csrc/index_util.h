// Pieces shared by the indexing translation units: a shape with magic-number dividers for decomposing a linear
// index, and the int32 / int64 index load.
#pragma once
#include <algorithm>

#include "common.h"

namespace tx {
namespace {

struct Dims {
  int n;
  FastDiv div[TX_MAX_DIMS];
  int64_t numel;
};

// a zero extent gets divider 1: such a shape has no elements and is never decomposed
inline void fill_dims(Dims* d, int nd, const int64_t* sizes) {
  d->n = nd;
  d->numel = 1;
  for (int i = 0; i < nd; ++i) {
    d->div[i] = FastDiv((uint32_t)std::min<int64_t>(std::max<int64_t>(sizes[i], 1), 0x7fffffff));
    d->numel *= sizes[i];
  }
}

__device__ __forceinline__ int64_t load_index(const char* p, int64_t off, int is64) {
  return is64 ? ((const int64_t*)p)[off] : (int64_t)((const int32_t*)p)[off];
}

}  // namespace
}  // namespace tx
