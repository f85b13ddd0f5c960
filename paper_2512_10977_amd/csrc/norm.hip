// layer_norm over the last k dims, and the fused sum / mean form of
// binary_cross_entropy (its elementwise form lives with the elementwise
// operators).
//
// layer_norm:
//   wave    : the normalised dims are contiguous in x, out, weight and bias and
//             a row fits 1024 16-byte vectors.  One wave64 owns a row and keeps
//             it in registers: one HBM read, mean, then the centred sum of
//             squares from the registers (two-pass variance without a second
//             read), one HBM write.
//   block   : the same with one 256-lane workgroup per row, for rows of up to
//             4096 vectors (16384 fp32 / 32768 half elements).
//   generic : anything else (longer rows, unaligned rows, strided normalised
//             dims).  One workgroup per row, three passes over the row with a
//             full index decomposition of the column; the re-reads hit L2.
// binary_cross_entropy, sum / mean: one pass; every workgroup reduces a chunk
//   of 4096 vectors to one binary64 partial, a second one-workgroup kernel adds
//   the partials, divides for the mean and rounds to the result dtype.
#include <cstring>

#include "common.h"
#include "loss.h"
#include "math_fp.h"
#include "rows.h"

namespace tx {
namespace {

// ---------------------------------------------------------------------------
// layer_norm
// ---------------------------------------------------------------------------
struct LnArgs {
  const char* x;
  char* out;
  const char* w;          // null: no weight
  const char* b;          // null: no bias
  int64_t rows, len;
  Slices lead;            // the leading dims: row -> offsets in x and out
  int w_f32, b_f32;       // weight / bias stored as fp32 although x is a half type
  int rows_per_group;     // consecutive rows taken by one workgroup (layer_norm_row_kernel) or wave
  float eps;
  // generic path: the normalised dims, inner-most last
  int inner_n;
  FastDiv idiv[TX_MAX_DIMS];
  int64_t ixs[TX_MAX_DIMS], ios[TX_MAX_DIMS], iws[TX_MAX_DIMS], ibs[TX_MAX_DIMS];
};

template <class T, int VEC> __device__ __forceinline__ void load_affine(const char* p, int f32, int64_t c, float (&o)[VEC]) {
  if (f32) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) o[e] = ((const float*)p)[c + e];
  } else {
    const Vec<T, VEC> t = vec_load<T, VEC, false>((const T*)p + c);
#pragma unroll
    for (int e = 0; e < VEC; ++e) o[e] = cvt<float>(t.v[e]);
  }
}

// BLOCK = false: one wave per row (four rows per workgroup); BLOCK = true: one workgroup per row.  Either way the
// owner keeps the row in registers, CH vectors of VEC elements per lane.
template <class T, int VEC, int CH, bool BLOCK>
__global__ __launch_bounds__(kBlock) void layer_norm_rows_kernel(const LnArgs a) {
  __shared__ float lds[kBlock / kWave];
  constexpr int kLanes = BLOCK ? kBlock : kWave;
  const int lane = BLOCK ? (int)threadIdx.x : (int)(threadIdx.x & (kWave - 1));
  const int64_t row = BLOCK ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * (kBlock / kWave) + (threadIdx.x / kWave);
  if constexpr (!BLOCK) {
    if (row >= a.rows) return;
  }
  int64_t xo, oo;
  slice_offsets(a.lead, row, &xo, &oo);
  const T* x = (const T*)a.x + xo;
  T* out = (T*)a.out + oo;
  float v[CH][VEC];
  float s = 0.0f;
  // loads in groups of up to 8, all unconditional (a vector past the row's end re-reads the first vector and
  // counts as zero), so that every load of a group is in flight before the first is used
  constexpr int kGroup = CH < 8 ? CH : 8;
#pragma unroll
  for (int k0 = 0; k0 < CH; k0 += kGroup) {
    Vec<T, VEC> t[kGroup];
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
      const int64_t c = ((int64_t)(k0 + j) * kLanes + lane) * VEC;
      t[j] = vec_load<T, VEC, true>(x + (c < a.len ? c : 0));
    }
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
      const int64_t c = ((int64_t)(k0 + j) * kLanes + lane) * VEC;
      const bool in = c < a.len;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        v[k0 + j][e] = in ? cvt<float>(t[j].v[e]) : 0.0f;
        s += v[k0 + j][e];
      }
    }
  }
  const float inv_len = 1.0f / (float)a.len;
  const float mean = (BLOCK ? block_reduce(s, false, lds) : wave_sum(s)) * inv_len;
  float sq = 0.0f;
#pragma unroll
  for (int k = 0; k < CH; ++k) {
    const int64_t c = ((int64_t)k * kLanes + lane) * VEC;
    const bool in = c < a.len;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      v[k][e] -= mean;
      sq += in ? v[k][e] * v[k][e] : 0.0f;
    }
  }
  const float rstd = 1.0f / sqrtf((BLOCK ? block_reduce(sq, false, lds) : wave_sum(sq)) * inv_len + a.eps);
#pragma unroll
  for (int k = 0; k < CH; ++k) {
    const int64_t c = ((int64_t)k * kLanes + lane) * VEC;
    if (c < a.len) {
      float w[VEC], b[VEC];
      if (a.w) load_affine<T, VEC>(a.w, a.w_f32, c, w);
      if (a.b) load_affine<T, VEC>(a.b, a.b_f32, c, b);
      Vec<T, VEC> t;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        float y = v[k][e] * rstd;
        if (a.w) y *= w[e];
        if (a.b) y += b[e];
        t.v[e] = cvt<T>(y);
      }
      vec_store<T, VEC, true>(out + c, t);
    }
  }
}

// A 256-lane workgroup per row, CH <= 4 vectors per lane (rows of 257 to 1024 vectors): a quarter of the registers
// of the wave-per-row form for the same row, so more resident waves.  The two workgroup-wide sums go through
// separate LDS slots (one barrier each).  A workgroup takes a.rows_per_group rows and fetches weight and
// bias once: fetched per row they are two more reads of the row's length from L2, which cost 23 us on [32768,4096]
// (192 us with them, 169 us - the time of a copy - without, one row per workgroup).  Each lane parks its own weight and bias vectors in LDS
// as it loaded them and reads them back per row (nobody else touches them, so no barrier is involved); held in
// registers instead they halve the resident waves).  Looping over rows costs a workgroup something by itself (183 us
// without weight and bias against 169 us for one row per workgroup), so the net gain is 192 -> 185 us for fp32 and
// 110 -> 98 us for bf16 on [32768,4096].
// Weight and bias have x's dtype here (fp32 parameters with a half x keep the wave form).
template <class T, int VEC, int CH>
__global__ __launch_bounds__(kBlock) void layer_norm_row_kernel(const LnArgs a) {
  constexpr int NW = kBlock / kWave;
  __shared__ float part_sum[NW], part_sq[NW];
  __shared__ __attribute__((aligned(16))) T lw[CH * kBlock * VEC], lb[CH * kBlock * VEC];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
#pragma unroll
  for (int k = 0; k < CH; ++k) {
    const int64_t c = ((int64_t)k * kBlock + threadIdx.x) * VEC;
    const int64_t cc = c < a.len ? c : 0;
    T* mine_w = lw + (k * kBlock + threadIdx.x) * VEC;
    T* mine_b = lb + (k * kBlock + threadIdx.x) * VEC;
    if (a.w) vec_store<T, VEC, false>(mine_w, vec_load<T, VEC, false>((const T*)a.w + cc));
    if (a.b) vec_store<T, VEC, false>(mine_b, vec_load<T, VEC, false>((const T*)a.b + cc));
  }
  const float inv_len = 1.0f / (float)a.len;
  // workgroup g takes rows g, g + G, g + 2 G, ... (G workgroups): the workgroups resident at one time then read one
  // contiguous window of the tensor, like a grid of one row per workgroup (with 8 consecutive rows per workgroup the
  // resident ones read 128 KiB apart, and the kernel took 210 us instead of 170 us)
  // (requesting the next row's vectors ahead, and a grid of four resident workgroups per CU, measured the same)
  for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
    int64_t xo, oo;
    slice_offsets(a.lead, row, &xo, &oo);
    const T* x = (const T*)a.x + xo;
    T* out = (T*)a.out + oo;
    Vec<T, VEC> t[CH];
#pragma unroll
    for (int k = 0; k < CH; ++k) {                              // all loads first, unconditional; len is a multiple of VEC here
      const int64_t c = ((int64_t)k * kBlock + threadIdx.x) * VEC;
      t[k] = vec_load<T, VEC, true>(x + (c < a.len ? c : 0));
    }
    float v[CH][VEC];
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < CH; ++k) {
      const bool in = ((int64_t)k * kBlock + threadIdx.x) * VEC < a.len;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        v[k][e] = in ? cvt<float>(t[k].v[e]) : 0.0f;
        s += v[k][e];
      }
    }
    s = wave_sum(s);
    if (lane == 0) part_sum[w] = s;
    __syncthreads();
    s = part_sum[0];
#pragma unroll
    for (int k = 1; k < NW; ++k) s += part_sum[k];
    const float mean = s * inv_len;
    float sq = 0.0f;
#pragma unroll
    for (int k = 0; k < CH; ++k) {
      const bool in = ((int64_t)k * kBlock + threadIdx.x) * VEC < a.len;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        v[k][e] -= mean;
        sq += in ? v[k][e] * v[k][e] : 0.0f;
      }
    }
    sq = wave_sum(sq);
    if (lane == 0) part_sq[w] = sq;
    __syncthreads();                        // also orders this row's reads of part_sum before the next row's writes
    sq = part_sq[0];
#pragma unroll
    for (int k = 1; k < NW; ++k) sq += part_sq[k];
    const float rstd = 1.0f / sqrtf(sq * inv_len + a.eps);
#pragma unroll
    for (int k = 0; k < CH; ++k) {
      const int64_t c = ((int64_t)k * kBlock + threadIdx.x) * VEC;
      if (c < a.len) {
        Vec<T, VEC> wv, bv, r;
        if (a.w) wv = vec_load<T, VEC, false>(lw + (k * kBlock + threadIdx.x) * VEC);
        if (a.b) bv = vec_load<T, VEC, false>(lb + (k * kBlock + threadIdx.x) * VEC);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          float y = v[k][e] * rstd;
          if (a.w) y *= cvt<float>(wv.v[e]);
          if (a.b) y += cvt<float>(bv.v[e]);
          r.v[e] = cvt<T>(y);
        }
        vec_store<T, VEC, true>(out + c, r);
      }
    }
  }
}

template <class T> __device__ __forceinline__ float load_affine1(const char* p, int f32, int64_t o) {
  return f32 ? ((const float*)p)[o] : cvt<float>(((const T*)p)[o]);
}

// one workgroup per row, three passes, any strides
template <class T>
__global__ __launch_bounds__(kBlock) void layer_norm_generic_kernel(const LnArgs a) {
  __shared__ float lds[kBlock / kWave];
  int64_t xo, oo;
  slice_offsets(a.lead, blockIdx.x, &xo, &oo);
  const T* x = (const T*)a.x + xo;
  T* out = (T*)a.out + oo;
  // column -> offsets in x / out / weight / bias
  auto offsets = [&](int64_t c, int64_t* px, int64_t* po, int64_t* pw, int64_t* pb) {
    int64_t ox = 0, oo2 = 0, ow = 0, ob = 0;
    uint32_t rem = (uint32_t)c;
    for (int d = a.inner_n - 1; d >= 0; --d) {
      uint32_t q, m;
      a.idiv[d].divmod(rem, q, m);
      rem = q;
      ox += (int64_t)m * a.ixs[d];
      oo2 += (int64_t)m * a.ios[d];
      ow += (int64_t)m * a.iws[d];
      ob += (int64_t)m * a.ibs[d];
    }
    *px = ox; *po = oo2; *pw = ow; *pb = ob;
  };
  float s = 0.0f;
  for (int64_t c = threadIdx.x; c < a.len; c += kBlock) {
    int64_t ox, o2, ow, ob;
    offsets(c, &ox, &o2, &ow, &ob);
    s += cvt<float>(x[ox]);
  }
  const float inv_len = 1.0f / (float)a.len;
  const float mean = block_reduce(s, false, lds) * inv_len;
  float sq = 0.0f;
  for (int64_t c = threadIdx.x; c < a.len; c += kBlock) {
    int64_t ox, o2, ow, ob;
    offsets(c, &ox, &o2, &ow, &ob);
    const float d = cvt<float>(x[ox]) - mean;
    sq += d * d;
  }
  const float rstd = 1.0f / sqrtf(block_reduce(sq, false, lds) * inv_len + a.eps);
  for (int64_t c = threadIdx.x; c < a.len; c += kBlock) {
    int64_t ox, o2, ow, ob;
    offsets(c, &ox, &o2, &ow, &ob);
    float y = (cvt<float>(x[ox]) - mean) * rstd;
    if (a.w) y *= load_affine1<T>(a.w, a.w_f32, ow);
    if (a.b) y += load_affine1<T>(a.b, a.b_f32, ob);
    out[o2] = cvt<T>(y);
  }
}

bool contiguous_tail(const tx_tensor* t, int d0) {
  int64_t expect = 1;
  for (int d = t->ndim - 1; d >= d0; --d) {
    if (t->sizes[d] != 1 && t->strides[d] != expect) return false;
    expect *= t->sizes[d];
  }
  return true;
}

template <class T>
tx_status layer_norm_launch(const tx_tensor* out, const tx_tensor* x, int lead, const tx_tensor* w, const tx_tensor* b,
                            double eps, hipStream_t stream) {
  constexpr int V = 16 / sizeof(T);
  LnArgs a;
  memset(&a, 0, sizeof(a));
  a.x = (const char*)x->data;
  a.out = (char*)out->data;
  a.w = w ? (const char*)w->data : nullptr;
  a.b = b ? (const char*)b->data : nullptr;
  a.w_f32 = w && w->dtype == TX_F32 && x->dtype != TX_F32;
  a.b_f32 = b && b->dtype == TX_F32 && x->dtype != TX_F32;
  a.eps = (float)eps;
  build_slices_range(&a.lead, x, out, 0, lead, -1);
  a.rows = a.lead.count;
  a.len = 1;
  for (int d = lead; d < x->ndim; ++d) a.len *= x->sizes[d];
  if (a.rows >= (1ll << 31) || a.len >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "layer_norm: too many rows / row too long");
  // the leading Slices must leave every row 16-byte aligned for the vector path
  bool aligned = (uintptr_t)x->data % 16 == 0 && (uintptr_t)out->data % 16 == 0 && a.len % V == 0;
  for (int d = 0; d < a.lead.n; ++d)
    aligned = aligned && (a.lead.xs[d] * (int64_t)sizeof(T)) % 16 == 0 && (a.lead.os[d] * (int64_t)sizeof(T)) % 16 == 0;
  if (w) aligned = aligned && (uintptr_t)w->data % 16 == 0;
  if (b) aligned = aligned && (uintptr_t)b->data % 16 == 0;
  const bool contig = contiguous_tail(x, lead) && contiguous_tail(out, lead) && (!w || contiguous_tail(w, 0)) &&
                      (!b || contiguous_tail(b, 0));
  const char* force = forced_path();
  const bool want_generic = !strcmp(force, "layer-norm-generic");
  const bool want_block = !strcmp(force, "layer-norm-block");
  // rows of more than 256 vectors (up to 1024): a workgroup per row with 2 or 4 vectors per lane, unless the wave form
  // is asked for by name
  const bool affine_like_x = (!w || w->dtype == x->dtype) && (!b || b->dtype == x->dtype);
  if (aligned && contig && a.len > 256 * V && a.len <= 1024 * V && affine_like_x && !want_generic && !want_block &&
      strcmp(force, "layer-norm-wave") != 0) {
    // as many rows per workgroup as still leave the chip 4096 workgroups (the weight and bias vectors are fetched once per workgroup)
    // as many rows per workgroup as still leave the chip 4096 workgroups (weight and bias are fetched once per workgroup)
    a.rows_per_group = a.rows >= 8 * 4096 ? 8 : a.rows >= 4 * 4096 ? 4 : a.rows >= 2 * 4096 ? 2 : 1;
    const dim3 grid((unsigned)((a.rows + a.rows_per_group - 1) / a.rows_per_group));
    set_path("layer-norm-row");
    if (a.len <= 512 * V) hipLaunchKernelGGL((layer_norm_row_kernel<T, V, 2>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((layer_norm_row_kernel<T, V, 4>), grid, dim3(kBlock), 0, stream, a);
    return check_launch("layer_norm row kernel");
  }
  if (aligned && contig && a.len <= 1024 * V && !want_generic && !want_block) {
    const dim3 grid((unsigned)((a.rows + 3) / 4));
    set_path("layer-norm-wave");
    if (a.len <= 64 * V) hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 1, false>), grid, dim3(kBlock), 0, stream, a);
    else if (a.len <= 128 * V) hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 2, false>), grid, dim3(kBlock), 0, stream, a);
    else if (a.len <= 256 * V) hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 4, false>), grid, dim3(kBlock), 0, stream, a);
    else if (a.len <= 512 * V) hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 8, false>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 16, false>), grid, dim3(kBlock), 0, stream, a);
    return check_launch("layer_norm wave kernel");
  }
  if (aligned && contig && a.len <= 4096 * V && !want_generic) {
    const dim3 grid((unsigned)a.rows);
    set_path("layer-norm-block");
    if (a.len <= 256 * V) hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 1, true>), grid, dim3(kBlock), 0, stream, a);
    else if (a.len <= 512 * V) hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 2, true>), grid, dim3(kBlock), 0, stream, a);
    else if (a.len <= 1024 * V) hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 4, true>), grid, dim3(kBlock), 0, stream, a);
    else if (a.len <= 2048 * V) hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 8, true>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((layer_norm_rows_kernel<T, V, 16, true>), grid, dim3(kBlock), 0, stream, a);
    return check_launch("layer_norm block kernel");
  }
  // generic: the normalised dims with every operand's strides (size-1 dims dropped)
  a.inner_n = 0;
  for (int d = lead; d < x->ndim; ++d) {
    if (x->sizes[d] == 1) continue;
    const int i = a.inner_n++;
    a.idiv[i] = FastDiv((uint32_t)x->sizes[d]);
    a.ixs[i] = x->strides[d];
    a.ios[i] = out->strides[d];
    a.iws[i] = w ? w->strides[d - lead] : 0;
    a.ibs[i] = b ? b->strides[d - lead] : 0;
  }
  set_path("layer-norm-generic");
  hipLaunchKernelGGL((layer_norm_generic_kernel<T>), dim3((unsigned)a.rows), dim3(kBlock), 0, stream, a);
  return check_launch("layer_norm generic kernel");
}

// ---------------------------------------------------------------------------
// binary_cross_entropy, sum / mean
// ---------------------------------------------------------------------------
constexpr int kBceUnroll = 4;

struct BceArgs {
  const char* x;
  const char* t;
  const char* w;            // mode 1: same layout as x; mode 2: one value per element of the last dim
  double* partial;
  int64_t n;                // elements
  int w_mode;               // 0 none, 1 same layout, 2 last-dim vector, 3: x already holds the losses
  int w_f32;
  FastDiv last;             // mode 2: extent of the last dim
  float param, half_param, half_over_param;   // KIND 3 / 4: beta or delta, half of it, 0.5 / it
};

// one term of the loss family.  KIND 0: binary_cross_entropy; 1: (x - t)^2; 2: |x - t|;
// 3: smooth_l1, |d| < beta ? d^2 / (2 beta) : |d| - beta / 2; 4: huber, |d| <= delta ? d^2 / 2 : delta (|d| - delta / 2).
// A NaN difference fails the comparison and comes out of the second form.
template <int KIND> __device__ __forceinline__ float loss_term(float x, float t, const BceArgs& a) {
  if constexpr (KIND == 0) return bce_term_fast(x, t);
  const float d = x - t, ad = __builtin_fabsf(d);
  if constexpr (KIND == 1) return d * d;
  if constexpr (KIND == 2) return ad;
  if constexpr (KIND == 3) return ad < a.param ? d * d * a.half_over_param : ad - a.half_param;
  return ad <= a.param ? 0.5f * d * d : a.param * (ad - a.half_param);
}

// MODE: the weight mode as a compile-time constant, or -1 = read a.w_mode at run time (the scalar kernel)
template <class T, int VEC, int MODE, int KIND = 0>
__global__ __launch_bounds__(kBlock) void bce_partial_kernel(const BceArgs a) {
  __shared__ double lds[kBlock / kWave];
  const int mode = MODE < 0 ? a.w_mode : MODE;
  const int64_t chunk = (int64_t)kBlock * VEC * kBceUnroll;
  const int64_t nchunks = (a.n + chunk - 1) / chunk;
  const T* x = (const T*)a.x;
  const T* t = (const T*)a.t;
  const int64_t last_vec = ((a.n - 1) / VEC) * VEC;      // n > 0; a ragged tail only exists for VEC == 1
  float acc = 0.0f;
  // the grid is capped, a workgroup takes chunks blockIdx.x, blockIdx.x + gridDim.x, ...: few partials for the
  // one-workgroup final kernel to add
  for (int64_t ch = blockIdx.x; ch < nchunks; ch += gridDim.x) {
    const int64_t base = ch * chunk + (int64_t)threadIdx.x * VEC;
    Vec<T, VEC> xv[kBceUnroll], tv[kBceUnroll];
#pragma unroll
    for (int u = 0; u < kBceUnroll; ++u) {
      const int64_t i = base + (int64_t)u * kBlock * VEC;
      const int64_t j = i < a.n ? i : last_vec;           // clamped: the load is unconditional
      xv[u] = vec_load<T, VEC, true>(x + j);
      if (mode != 3) tv[u] = vec_load<T, VEC, true>(t + j);
    }
#pragma unroll
    for (int u = 0; u < kBceUnroll; ++u) {
      const int64_t i = base + (int64_t)u * kBlock * VEC;
      if (i < a.n) {
        // the weights of one vector of x are one aligned vector themselves (mode 2: last % VEC == 0, so a vector
        // never straddles two rows; n < 2^31)
        float wv[VEC];
        if (mode == 1) load_affine<T, VEC>(a.w, a.w_f32, i, wv);
        if (mode == 2) {
          uint32_t q, m;
          a.last.divmod((uint32_t)i, q, m);
          load_affine<T, VEC>(a.w, a.w_f32, m, wv);
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          float l = mode == 3 ? cvt<float>(xv[u].v[e]) : loss_term<KIND>(cvt<float>(xv[u].v[e]), cvt<float>(tv[u].v[e]), a);
          if (mode == 1 || mode == 2) l *= wv[e];
          acc += l;
        }
      }
    }
  }
  double d = (double)acc;
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) d += shfl_xor(d, m);
  if ((threadIdx.x & (kWave - 1)) == 0) lds[threadIdx.x / kWave] = d;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < kBlock / kWave; ++k) s += lds[k];
    a.partial[blockIdx.x] = s;
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void bce_final_kernel(const double* partial, int64_t count, int64_t n, int mean, T* out) {
  __shared__ double lds[kBlock / kWave];
  double d = 0.0;
  for (int64_t i = threadIdx.x; i < count; i += kBlock) d += partial[i];
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) d += shfl_xor(d, m);
  if ((threadIdx.x & (kWave - 1)) == 0) lds[threadIdx.x / kWave] = d;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < kBlock / kWave; ++k) s += lds[k];
    if (mean) s = s / (double)n;                       // 0 / 0 = NaN: the mean of no elements
    *out = cvt<T>((float)s);
  }
}

// same strides, and the strides describe a dense block of memory (any dim order): a sum over all elements may
// then walk memory linearly
bool dense_same_layout(const tx_tensor* x, const tx_tensor* y) {
  if (x->ndim != y->ndim) return false;
  for (int d = 0; d < x->ndim; ++d)
    if (x->sizes[d] != y->sizes[d] || (x->sizes[d] != 1 && x->strides[d] != y->strides[d])) return false;
  int order[TX_MAX_DIMS], n = 0;
  for (int d = 0; d < x->ndim; ++d)
    if (x->sizes[d] != 1) order[n++] = d;
  std::sort(order, order + n, [&](int p, int q) { return x->strides[p] < x->strides[q]; });
  int64_t expect = 1;
  for (int i = 0; i < n; ++i) {
    if (x->strides[order[i]] != expect) return false;
    expect *= x->sizes[order[i]];
  }
  return true;
}

}  // namespace

// how the fused kernel can read the operands: -1 = it cannot (the caller forms the losses first), else the weight mode
int bce_fused_mode(const tx_tensor* x, const tx_tensor* t, const tx_tensor* w) {
  if (!dense_same_layout(x, t)) return -1;
  if (!w) return 0;
  if (w->dtype != x->dtype && w->dtype != TX_F32) return -1;
  if (w->ndim == x->ndim && dense_same_layout(x, w)) return 1;
  // one weight per element of the last dim, x row-major
  if (x->ndim >= 1 && numel(x) < (1ll << 31) && contiguous_tail(x, 0) && numel(w) == x->sizes[x->ndim - 1] && w->ndim >= 1 &&
      w->sizes[w->ndim - 1] == numel(w) && (numel(w) == 1 || w->strides[w->ndim - 1] == 1))
    return 2;
  return -1;
}

constexpr int64_t kBceMaxBlocks = 2048;                 // 8 workgroups per compute unit
size_t bce_partial_count(int64_t n, int esize) {
  const int64_t chunk = (int64_t)kBlock * (16 / esize) * kBceUnroll;
  return (size_t)std::min<int64_t>((n + chunk - 1) / chunk, kBceMaxBlocks);
}

// sum / mean of the losses.  mode 3: `x` holds precomputed losses (contiguous, n elements)
template <class T>
tx_status bce_reduce_typed(const tx_tensor* out, const void* x, const void* t, const tx_tensor* w, int mode, int64_t n,
                           int64_t last, int mean, double* partial, hipStream_t stream, int kind, double param) {
  constexpr int V = 16 / sizeof(T);
  size_t blocks = 0;
  if (n > 0) {
    BceArgs a;
    memset(&a, 0, sizeof(a));
    a.x = (const char*)x;
    a.t = (const char*)t;
    a.w = w ? (const char*)w->data : nullptr;
    a.partial = partial;
    a.n = n;
    a.w_mode = mode;
    a.w_f32 = w && w->dtype == TX_F32 && sizeof(T) == 2;
    a.last = FastDiv((uint32_t)std::max<int64_t>(1, std::min<int64_t>(last, 0x7fffffff)));
    a.param = (float)param;
    a.half_param = (float)(0.5 * param);
    a.half_over_param = (float)(0.5 / param);          // beta = 0: infinite and never selected
    blocks = bce_partial_count(n, sizeof(T));
    bool al = (uintptr_t)x % 16 == 0 && (mode == 3 || (uintptr_t)t % 16 == 0) && n % V == 0;
    if (mode == 1 || mode == 2) al = al && (uintptr_t)w->data % 16 == 0 && (mode == 1 || last % V == 0);
    if (kind != 0 && mode != 3) {                      // the regression losses: no weight
      const dim3 grid((unsigned)(al ? blocks : std::min<int64_t>((n + kBlock * kBceUnroll - 1) / (kBlock * kBceUnroll), kBceMaxBlocks)));
      if (!al) blocks = grid.x;
      set_path(al ? "loss-fused" : "loss-fused-scalar");
      auto go = [&](auto k) {
        constexpr int K = decltype(k)::value;
        if (al) hipLaunchKernelGGL((bce_partial_kernel<T, V, 0, K>), grid, dim3(kBlock), 0, stream, a);
        else hipLaunchKernelGGL((bce_partial_kernel<T, 1, -1, K>), grid, dim3(kBlock), 0, stream, a);
      };
      switch (kind) {
        case 1: go(std::integral_constant<int, 1>{}); break;
        case 2: go(std::integral_constant<int, 2>{}); break;
        case 3: go(std::integral_constant<int, 3>{}); break;
        default: go(std::integral_constant<int, 4>{}); break;
      }
    } else if (al) {
      const dim3 grid((unsigned)blocks);
      set_path("bce-fused");
      switch (mode) {
        case 0: hipLaunchKernelGGL((bce_partial_kernel<T, V, 0>), grid, dim3(kBlock), 0, stream, a); break;
        case 1: hipLaunchKernelGGL((bce_partial_kernel<T, V, 1>), grid, dim3(kBlock), 0, stream, a); break;
        case 2: hipLaunchKernelGGL((bce_partial_kernel<T, V, 2>), grid, dim3(kBlock), 0, stream, a); break;
        default: hipLaunchKernelGGL((bce_partial_kernel<T, V, 3>), grid, dim3(kBlock), 0, stream, a); break;
      }
    } else {
      blocks = (size_t)std::min<int64_t>((n + kBlock * kBceUnroll - 1) / (kBlock * kBceUnroll), kBceMaxBlocks);
      set_path("bce-fused-scalar");
      hipLaunchKernelGGL((bce_partial_kernel<T, 1, -1>), dim3((unsigned)blocks), dim3(kBlock), 0, stream, a);
    }
    tx_status rc = check_launch("binary_cross_entropy partial kernel");
    if (rc) return rc;
  } else {
    set_path("bce-fused");
  }
  hipLaunchKernelGGL((bce_final_kernel<T>), dim3(1), dim3(kBlock), 0, stream, partial, (int64_t)blocks, n, mean, (T*)out->data);
  return check_launch("binary_cross_entropy final kernel");
}

tx_status bce_reduce(const tx_tensor* out, int dtype, const void* x, const void* t, const tx_tensor* w, int mode, int64_t n,
                     int64_t last, int mean, double* partial, hipStream_t stream, int kind, double param) {
  switch (dtype) {
    case TX_F32: return bce_reduce_typed<float>(out, x, t, w, mode, n, last, mean, partial, stream, kind, param);
    case TX_BF16: return bce_reduce_typed<bf16>(out, x, t, w, mode, n, last, mean, partial, stream, kind, param);
    default: return bce_reduce_typed<f16>(out, x, t, w, mode, n, last, mean, partial, stream, kind, param);
  }
}

}  // namespace tx

using namespace tx;

extern "C" {

tx_status tx_layer_norm(const tx_tensor* out, const tx_tensor* x, int32_t norm_ndim, const tx_tensor* weight,
                        const tx_tensor* bias, double eps, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x"))) return rc;
  if (weight && (rc = check_tensor(weight, "weight"))) return rc;
  if (bias && (rc = check_tensor(bias, "bias"))) return rc;
  if (!dtype_is_float(x->dtype)) return fail(TX_ERR_DTYPE, "layer_norm takes floating dtypes only");
  if (out->dtype != x->dtype) return fail(TX_ERR_DTYPE, "layer_norm: out must have x's dtype");
  if ((weight && !dtype_is_float(weight->dtype)) || (bias && !dtype_is_float(bias->dtype)))
    return fail(TX_ERR_DTYPE, "layer_norm: weight / bias must be floating");
  if (!same_sizes(out, x->ndim, x->sizes)) return fail(TX_ERR_SHAPE, "layer_norm: out must have x's shape");
  if (norm_ndim < 1 || norm_ndim > x->ndim) return fail(TX_ERR_DIM, "layer_norm: %d normalised dims for a %d-dim input", norm_ndim, x->ndim);
  const int lead = x->ndim - norm_ndim;
  if (weight && !same_sizes(weight, norm_ndim, x->sizes + lead)) return fail(TX_ERR_SHAPE, "layer_norm: weight shape");
  if (bias && !same_sizes(bias, norm_ndim, x->sizes + lead)) return fail(TX_ERR_SHAPE, "layer_norm: bias shape");
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  const tx_tensor* ins[3] = {x, weight, bias};
  for (const tx_tensor* in : ins)
    if (in && (partial_overlap(out, in) || (out->data == in->data && numel(in) > 0)))
      return fail(TX_ERR_OVERLAP, "layer_norm: out must not alias an input");
  // kernels read weight / bias as x's dtype or fp32
  for (const tx_tensor* in : {weight, bias})
    if (in && in->dtype != x->dtype && in->dtype != TX_F32)
      return fail(TX_ERR_UNSUPPORTED, "layer_norm: weight / bias must have x's dtype or fp32");
  set_path("");
  if (numel(x) == 0) return TX_OK;
  hipStream_t s = as_stream(stream);
  switch (x->dtype) {
    case TX_F32: return layer_norm_launch<float>(out, x, lead, weight, bias, eps, s);
    case TX_BF16: return layer_norm_launch<bf16>(out, x, lead, weight, bias, eps, s);
    default: return layer_norm_launch<f16>(out, x, lead, weight, bias, eps, s);
  }
}

}  // extern "C"
