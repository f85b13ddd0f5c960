// Helpers shared by the row-wise translation units (softmax / cumsum, layer_norm): the collapsed set of "other"
// dims that enumerates rows, and wave / workgroup reductions.
#pragma once
#include <algorithm>

#include "common.h"

namespace tx {

// column forms (colops.hip): the operated dim is not the innermost one and the dims after it are one contiguous run
bool cols_path_ok(const tx_tensor* out, const tx_tensor* x, int dim);
tx_status softmax_cols(const tx_tensor* out, const tx_tensor* x, int dim, int is_log, hipStream_t stream);
tx_status cumsum_cols(const tx_tensor* out, const tx_tensor* x, int dim, void* ws, size_t ws_bytes, hipStream_t stream,
                      size_t* query);

namespace {

constexpr int kBlock = 256;

// the dims other than `dim`, merged where both tensors allow, inner-most last
struct Slices {
  int n;
  FastDiv div[TX_MAX_DIMS];
  int64_t size[TX_MAX_DIMS], xs[TX_MAX_DIMS], os[TX_MAX_DIMS];
  int64_t count;
};

// dims [d0, d1) of x / out except `skip`
inline void build_slices_range(Slices* s, const tx_tensor* x, const tx_tensor* out, int d0, int d1, int skip) {
  s->n = 0;
  s->count = 1;
  for (int d = d0; d < d1; ++d) {
    if (d == skip) continue;
    const int64_t sz = x->sizes[d];
    s->count *= sz;
    if (sz == 1) continue;
    if (s->n > 0 && s->xs[s->n - 1] == x->strides[d] * sz && s->os[s->n - 1] == out->strides[d] * sz) {
      s->size[s->n - 1] *= sz;
      s->xs[s->n - 1] = x->strides[d];
      s->os[s->n - 1] = out->strides[d];
    } else {
      s->size[s->n] = sz;
      s->xs[s->n] = x->strides[d];
      s->os[s->n] = out->strides[d];
      ++s->n;
    }
  }
  for (int d = 0; d < s->n; ++d) s->div[d] = FastDiv((uint32_t)std::min<int64_t>(s->size[d], 0x7fffffff));
}

inline void build_slices(Slices* s, const tx_tensor* x, const tx_tensor* out, int dim) {
  build_slices_range(s, x, out, 0, x->ndim, dim);
}

__device__ __forceinline__ void slice_offsets(const Slices& s, int64_t idx, int64_t* xo, int64_t* oo) {
  int64_t x = 0, o = 0;
  if (s.n == 1) { x = idx * s.xs[0]; o = idx * s.os[0]; }
  else {
    uint32_t rem = (uint32_t)idx;
    for (int d = s.n - 1; d >= 0; --d) {
      uint32_t q, m;
      s.div[d].divmod(rem, q, m);
      rem = q;
      x += (int64_t)m * s.xs[d];
      o += (int64_t)m * s.os[d];
    }
  }
  *xo = x;
  *oo = o;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) v = fmaxf(v, shfl_xor(v, m));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) v += shfl_xor(v, m);
  return v;
}
constexpr float kNegInf = -__builtin_huge_valf();

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* lds) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int w = threadIdx.x / kWave;
  __syncthreads();                          // protects lds reuse between calls
  if ((threadIdx.x & (kWave - 1)) == 0) lds[w] = v;
  __syncthreads();
  float r = lds[0];
#pragma unroll
  for (int k = 1; k < kBlock / kWave; ++k) r = is_max ? fmaxf(r, lds[k]) : r + lds[k];
  return r;
}

// one lane per slice: the slices, and the extent and strides of the dim operated on
struct StridedArgs {
  const char* x;
  char* out;
  Slices sl;
  int64_t len, xs, os;
  int is_log;
};

}  // namespace
}  // namespace tx
