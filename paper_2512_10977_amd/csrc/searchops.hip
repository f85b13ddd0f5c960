// searchsorted / bucketize: one lane per value bisects its sorted row.
//
// The probes of the first levels are the same addresses for every lane of a row and stay in cache; the last levels
// are scattered 4- or 8-byte reads, so the operator is bound by the value read and the index write only while the
// sequence fits the caches.  Each lane carries kSearchU independent searches so that their probes overlap.
#include <cstring>

#include "common.h"
#include "index_util.h"

namespace tx {
namespace {

constexpr int kBlock = 256;
constexpr int kSearchU = 4;

struct SearchArgs {
  Dims shape;                        // values' (= out's) shape
  int64_t vstride[TX_MAX_DIMS], ostride[TX_MAX_DIMS];
  int64_t qstride[TX_MAX_DIMS];      // the sequence's strides over the leading dims (all 0 for a 1-D sequence)
  int64_t qlast;                     // its stride along the searched dim
  int64_t n;                         // elements per sequence row
  const char* seq;
  const char* values;
  char* out;
  int right, out64;
};

template <class T> struct SearchKey { using type = T; };
template <> struct SearchKey<bf16> { using type = float; };          // the conversions are exact and keep the order
template <> struct SearchKey<f16> { using type = float; };

template <class T>
__global__ __launch_bounds__(kBlock) void searchsorted_kernel(const SearchArgs a) {
  using K = typename SearchKey<T>::type;
  int64_t qo[kSearchU], d_o[kSearchU];
  int64_t start[kSearchU], end[kSearchU];
  K v[kSearchU];
  bool live[kSearchU];
#pragma unroll
  for (int u = 0; u < kSearchU; ++u) {
    const int64_t lin = ((int64_t)blockIdx.x * kSearchU + u) * kBlock + threadIdx.x;
    live[u] = lin < a.shape.numel;
    qo[u] = d_o[u] = 0;
    start[u] = end[u] = 0;
    v[u] = K(0);
    if (!live[u]) continue;
    int64_t vo = 0;
    uint32_t rem = (uint32_t)lin;
    for (int d = a.shape.n - 1; d >= 0; --d) {
      uint32_t q, m;
      a.shape.div[d].divmod(rem, q, m);
      rem = q;
      vo += (int64_t)m * a.vstride[d];
      d_o[u] += (int64_t)m * a.ostride[d];
      qo[u] += (int64_t)m * a.qstride[d];
    }
    v[u] = cvt<K>(((const T*)a.values)[vo]);
    end[u] = a.n;
  }
  // bisection of [start, end): move right while the probed element does not yet satisfy the stopping comparison (a
  // NaN value never stops, a NaN element never stops either).  Every search of the lane takes one step per round.
  bool any = true;
  while (any) {
    any = false;
#pragma unroll
    for (int u = 0; u < kSearchU; ++u) {
      if (start[u] < end[u]) {
        const int64_t mid = start[u] + ((end[u] - start[u]) >> 1);
        const K e = cvt<K>(((const T*)a.seq)[qo[u] + mid * a.qlast]);
        const bool stop = a.right ? e > v[u] : e >= v[u];
        if (!stop) start[u] = mid + 1;
        else end[u] = mid;
        any = any || start[u] < end[u];
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kSearchU; ++u) {
    if (!live[u]) continue;
    if (a.out64) ((int64_t*)a.out)[d_o[u]] = start[u];
    else ((int32_t*)a.out)[d_o[u]] = (int32_t)start[u];
  }
}

// The same search for a 1-D sequence shared by every value: the probes of the first kTreeLevels levels are the same
// few addresses for every value, so each workgroup first copies them into LDS in heap order (slot 1 is the first
// midpoint, slots 2k and 2k + 1 the midpoints after going left / right from slot k) and walks that copy; only the
// remaining levels probe memory.  The steps, and so the results, are those of the plain bisection on any input.
constexpr int kTreeLevels = 10;             // 1023 slots (12 levels measured no faster: the walk itself is the cost)
constexpr int kTreeSlots = 1 << kTreeLevels;
constexpr int kTreeMinLength = 2 * kTreeSlots;        // every interval of the first levels is non-empty from here on

template <class T>
__global__ __launch_bounds__(kBlock) void searchsorted_tree_kernel(const SearchArgs a, int tiles_per_wg) {
  using K = typename SearchKey<T>::type;
  __shared__ K tree[kTreeSlots];
  for (int k = threadIdx.x + 1; k < kTreeSlots; k += kBlock) {
    const int level = 31 - __clz(k);
    int64_t start = 0, end = a.n;
    for (int b = level - 1; b >= 0; --b) {
      const int64_t mid = start + ((end - start) >> 1);
      if ((k >> b) & 1) start = mid + 1;
      else end = mid;
    }
    K e = K(0);
    if (start < end) e = cvt<K>(((const T*)a.seq)[(start + ((end - start) >> 1)) * a.qlast]);
    tree[k] = e;
  }
  __syncthreads();
  for (int t = 0; t < tiles_per_wg; ++t) {
    const int64_t tile = (int64_t)blockIdx.x * tiles_per_wg + t;
    int64_t d_o[kSearchU], start[kSearchU], end[kSearchU];
    K v[kSearchU];
    bool live[kSearchU];
#pragma unroll
    for (int u = 0; u < kSearchU; ++u) {
      const int64_t lin = (tile * kSearchU + u) * kBlock + threadIdx.x;
      live[u] = lin < a.shape.numel;
      d_o[u] = 0;
      start[u] = end[u] = 0;
      v[u] = K(0);
      if (!live[u]) continue;
      int64_t vo = 0;
      uint32_t rem = (uint32_t)lin;
      for (int d = a.shape.n - 1; d >= 0; --d) {
        uint32_t q, m;
        a.shape.div[d].divmod(rem, q, m);
        rem = q;
        vo += (int64_t)m * a.vstride[d];
        d_o[u] += (int64_t)m * a.ostride[d];
      }
      v[u] = cvt<K>(((const T*)a.values)[vo]);
      end[u] = a.n;
      int k = 1;
      for (int l = 0; l < kTreeLevels; ++l) {              // intervals of these levels are never empty
        const int64_t mid = start[u] + ((end[u] - start[u]) >> 1);
        const K e = tree[k];
        const bool stop = a.right ? e > v[u] : e >= v[u];
        if (!stop) start[u] = mid + 1;
        else end[u] = mid;
        k = 2 * k + (stop ? 0 : 1);
      }
    }
    bool any = true;
    while (any) {
      any = false;
#pragma unroll
      for (int u = 0; u < kSearchU; ++u) {
        if (start[u] < end[u]) {
          const int64_t mid = start[u] + ((end[u] - start[u]) >> 1);
          const K e = cvt<K>(((const T*)a.seq)[mid * a.qlast]);
          const bool stop = a.right ? e > v[u] : e >= v[u];
          if (!stop) start[u] = mid + 1;
          else end[u] = mid;
          any = any || start[u] < end[u];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kSearchU; ++u) {
      if (!live[u]) continue;
      if (a.out64) ((int64_t*)a.out)[d_o[u]] = start[u];
      else ((int32_t*)a.out)[d_o[u]] = (int32_t)start[u];
    }
  }
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

tx_status tx_searchsorted(const tx_tensor* out, const tx_tensor* sorted_sequence, const tx_tensor* values, int right, void* stream) {
  tx_status rc;
  const tx_tensor* seq = sorted_sequence;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(seq, "sorted_sequence")) || (rc = check_tensor(values, "values"))) return rc;
  if (seq->dtype != values->dtype) return fail(TX_ERR_DTYPE, "searchsorted: the sequence and the values must have one dtype");
  if (seq->dtype == TX_BOOL) return fail(TX_ERR_DTYPE, "searchsorted does not take bool");
  if (out->dtype != TX_I64 && out->dtype != TX_I32) return fail(TX_ERR_DTYPE, "searchsorted: out must be int64 or int32");
  if (seq->ndim < 1) return fail(TX_ERR_NDIM, "searchsorted: the sequence needs at least one dim");
  if (seq->ndim != 1) {
    if (seq->ndim != values->ndim) return fail(TX_ERR_SHAPE, "searchsorted: an N-D sequence needs values of the same rank");
    for (int d = 0; d + 1 < seq->ndim; ++d)
      if (seq->sizes[d] != values->sizes[d]) return fail(TX_ERR_SHAPE, "searchsorted: leading dims of the sequence and the values differ");
  }
  if (!same_sizes(out, values->ndim, values->sizes)) return fail(TX_ERR_SHAPE, "searchsorted: out must have the values' shape");
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  const int64_t m = numel(out);
  if (m && ((numel(seq) && (partial_overlap(out, seq) || out->data == seq->data)) || partial_overlap(out, values) ||
            (out->data == values->data)))
    return fail(TX_ERR_OVERLAP, "searchsorted: out overlaps an input");
  set_path("");
  if (m == 0) return TX_OK;
  if (m >= (1ll << 31) || numel(seq) >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "searchsorted: more than 2^31 elements");
  SearchArgs a;
  memset(&a, 0, sizeof(a));
  fill_dims(&a.shape, values->ndim, values->sizes);
  for (int d = 0; d < values->ndim; ++d) {
    a.vstride[d] = values->strides[d];
    a.ostride[d] = out->strides[d];
    a.qstride[d] = (seq->ndim != 1 && d + 1 < seq->ndim) ? seq->strides[d] : 0;
  }
  a.qlast = seq->strides[seq->ndim - 1];
  a.n = seq->sizes[seq->ndim - 1];
  a.seq = (const char*)seq->data;
  a.values = (const char*)values->data;
  a.out = (char*)out->data;
  a.right = right != 0;
  a.out64 = out->dtype == TX_I64;
  hipStream_t s = as_stream(stream);
  if (seq->ndim == 1 && a.n >= kTreeMinLength && m >= (1 << 16) && strcmp(forced_path(), "searchsorted")) {
    const int tiles_per_wg = 8;                         // the tree is built once per workgroup
    const int64_t per_wg = (int64_t)kBlock * kSearchU * tiles_per_wg;
    const dim3 tgrid((unsigned)((m + per_wg - 1) / per_wg));
    set_path("searchsorted-tree");
    switch (seq->dtype) {
      case TX_F32: hipLaunchKernelGGL((searchsorted_tree_kernel<float>), tgrid, dim3(kBlock), 0, s, a, tiles_per_wg); break;
      case TX_BF16: hipLaunchKernelGGL((searchsorted_tree_kernel<bf16>), tgrid, dim3(kBlock), 0, s, a, tiles_per_wg); break;
      case TX_F16: hipLaunchKernelGGL((searchsorted_tree_kernel<f16>), tgrid, dim3(kBlock), 0, s, a, tiles_per_wg); break;
      case TX_I32: hipLaunchKernelGGL((searchsorted_tree_kernel<int32_t>), tgrid, dim3(kBlock), 0, s, a, tiles_per_wg); break;
      default: hipLaunchKernelGGL((searchsorted_tree_kernel<int64_t>), tgrid, dim3(kBlock), 0, s, a, tiles_per_wg); break;
    }
    return check_launch("searchsorted tree kernel");
  }
  const dim3 grid((unsigned)((m + kBlock * kSearchU - 1) / (kBlock * kSearchU)));
  set_path("searchsorted");
  switch (seq->dtype) {
    case TX_F32: hipLaunchKernelGGL((searchsorted_kernel<float>), grid, dim3(kBlock), 0, s, a); break;
    case TX_BF16: hipLaunchKernelGGL((searchsorted_kernel<bf16>), grid, dim3(kBlock), 0, s, a); break;
    case TX_F16: hipLaunchKernelGGL((searchsorted_kernel<f16>), grid, dim3(kBlock), 0, s, a); break;
    case TX_I32: hipLaunchKernelGGL((searchsorted_kernel<int32_t>), grid, dim3(kBlock), 0, s, a); break;
    default: hipLaunchKernelGGL((searchsorted_kernel<int64_t>), grid, dim3(kBlock), 0, s, a); break;
  }
  return check_launch("searchsorted kernel");
}

}  // extern "C"
