// softmax / log_softmax and cumsum along a dim that is NOT the innermost one,
// for tensors whose dims after it form one contiguous run ("columns"): the
// tensor is seen as [outer..., L, inner] with inner contiguous.  Lanes run
// along `inner` (coalesced), the operated dim is walked with its stride.
//
// softmax : a 1024-lane workgroup owns a strip of columns; its 16 waves take
//           interleaved rows and keep a running (max, scaled sum) per column,
//           merge through LDS, then read the strip again and write.  Two
//           reads and one write per element.
// cumsum  : the rows are cut into tiles.  Pass A sums every tile per column
//           into the workspace, pass B turns those sums into exclusive
//           prefixes (in place), pass C scans every tile from registers,
//           adds its prefix and writes.  Two reads and one write per element;
//           with a single tile per column passes A and B are skipped.
#include <cstring>

#include "common.h"
#include "rows.h"

namespace tx {
namespace {

constexpr int kColWaves = 16;                 // softmax: waves per workgroup
constexpr int kColBlock = kColWaves * kWave;

struct ColArgs {
  const char* x;
  char* out;
  Slices outer;             // the dims before the operated one
  int64_t L, inner, xs, os; // extent and strides of the operated dim, extent of the contiguous run after it
  int64_t col_tiles;        // column strips per outer slice
  int is_log;
  // cumsum
  char* ws;
  int64_t tiles_l, rows_per_block;
};

// running (m, s) with s = sum exp(x - m): one hardware exp per element, no branches.  m starts at -inf with s = 0;
// exp(-inf) = 0 covers that state and +inf elements; a NaN element makes s NaN for good (m ignores it).
__device__ __forceinline__ void ms_step(float& m, float& s, float v) {
  const float d = v == m ? 0.0f : -__builtin_fabsf(v - m);
  const float e = __expf(d);
  const bool le = v <= m;
  s = __builtin_fmaf(e, le ? 1.0f : s, le ? s : 1.0f);
  m = __builtin_fmaxf(m, v);
}
__device__ __forceinline__ void ms_merge(float& m, float& s, float m2, float s2) {
  const float M = __builtin_fmaxf(m, m2);
  const float e1 = m == M ? 1.0f : __expf(m - M), e2 = m2 == M ? 1.0f : __expf(m2 - M);
  s = s * e1 + s2 * e2;
  m = M;
}

// VEC columns per lane, CPW column-lanes per wave (the other 64 / CPW lanes of a wave take further rows)
template <class T, class O, int VEC, int CPW>
__global__ __launch_bounds__(kColBlock) void softmax_cols_kernel(const ColArgs a) {
  constexpr int RL = kWave / CPW, CW = CPW * VEC, RS = kColWaves * RL, U = 4;
  __shared__ float lm[kColWaves][CW], ls[kColWaves][CW];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int cl = lane % CPW, rl = lane / CPW;
  const int64_t tile = blockIdx.x % a.col_tiles, o = blockIdx.x / a.col_tiles;
  int64_t xo, oo;
  slice_offsets(a.outer, o, &xo, &oo);
  const int64_t col = tile * CW + (int64_t)cl * VEC;
  const bool active = col < a.inner;                       // inner is a multiple of VEC when VEC > 1
  const T* xp = (const T*)a.x + xo + (active ? col : 0);
  O* op = (O*)a.out + oo + (active ? col : 0);
  const int64_t r0 = (int64_t)w * RL + rl;
  float m[VEC], s[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { m[e] = kNegInf; s[e] = 0.0f; }
  // U rows per step, every load unconditional (a row past the end re-reads the last row and is not used)
  for (int64_t l = r0; l < a.L; l += (int64_t)RS * U) {
    Vec<T, VEC> t[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const int64_t lk = l + (int64_t)k * RS;
      t[k] = vec_load<T, VEC, false>(xp + (lk < a.L ? lk : a.L - 1) * a.xs);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      if (l + (int64_t)k * RS < a.L) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) ms_step(m[e], s[e], cvt<float>(t[k].v[e]));
      }
    }
  }
#pragma unroll
  for (int sh = CPW; sh < kWave; sh <<= 1) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) ms_merge(m[e], s[e], shfl_xor(m[e], sh), shfl_xor(s[e], sh));
  }
  if (rl == 0) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) { lm[w][cl * VEC + e] = m[e]; ls[w][cl * VEC + e] = s[e]; }
  }
  __syncthreads();
  float inv[VEC], lg[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    float M = lm[0][cl * VEC + e], S = ls[0][cl * VEC + e];
#pragma unroll
    for (int ww = 1; ww < kColWaves; ++ww) ms_merge(M, S, lm[ww][cl * VEC + e], ls[ww][cl * VEC + e]);
    if (M == -kNegInf) S = __uint_as_float(0x7fc00000u);   // a +inf element: inf - inf, every output is NaN
    m[e] = M;
    inv[e] = 1.0f / S;
    lg[e] = logf(S);
  }
  for (int64_t l = r0; l < a.L; l += (int64_t)RS * U) {
    Vec<T, VEC> t[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const int64_t lk = l + (int64_t)k * RS;
      t[k] = vec_load<T, VEC, true>(xp + (lk < a.L ? lk : a.L - 1) * a.xs);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const int64_t lk = l + (int64_t)k * RS;
      if (lk < a.L && active) {
        Vec<O, VEC> r;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float d = cvt<float>(t[k].v[e]) - m[e];
          r.v[e] = cvt<O>(a.is_log ? d - lg[e] : expf(d) * inv[e]);
        }
        vec_store<O, VEC, true>(op + lk * a.os, r);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// cumsum
// ---------------------------------------------------------------------------
constexpr int kScanWaves = kBlock / kWave;    // 4
constexpr int kScanRows = 16;                  // rows per wave per step
constexpr int kScanStep = kScanWaves * kScanRows;

template <class T, class Acc, int VEC>
__device__ __forceinline__ void col_block(const ColArgs& a, int64_t* o, int64_t* tl, int64_t* row0, int64_t* row1,
                                          int64_t* col, bool* active) {
  const int64_t b = blockIdx.x;
  const int64_t tile = b % a.col_tiles;
  *tl = (b / a.col_tiles) % a.tiles_l;
  *o = b / (a.col_tiles * a.tiles_l);
  *row0 = *tl * a.rows_per_block;
  *row1 = *row0 + a.rows_per_block < a.L ? *row0 + a.rows_per_block : a.L;
  *col = tile * (int64_t)(kWave * VEC) + (int64_t)(threadIdx.x & (kWave - 1)) * VEC;
  *active = *col < a.inner;
}

// pass A: per tile and column, the sum of the tile's rows -> ws[(o * tiles_l + tl) * inner + col]
template <class T, class Acc, int VEC>
__global__ __launch_bounds__(kBlock) void colscan_sums_kernel(const ColArgs a) {
  __shared__ Acc tot[kScanWaves][kWave * VEC];
  int64_t o, tl, row0, row1, col;
  bool active;
  col_block<T, Acc, VEC>(a, &o, &tl, &row0, &row1, &col, &active);
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  int64_t xo, oo;
  slice_offsets(a.outer, o, &xo, &oo);
  const T* xp = (const T*)a.x + xo + (active ? col : 0);
  Acc acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = Acc(0);
  constexpr int U = 8;
  for (int64_t l = row0 + w; l < row1; l += kScanWaves * U) {
    Vec<T, VEC> t[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const int64_t lk = l + k * kScanWaves;
      t[k] = vec_load<T, VEC, false>(xp + (lk < row1 ? lk : row1 - 1) * a.xs);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      if (l + k * kScanWaves < row1) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += cvt<Acc>(t[k].v[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) tot[w][lane * VEC + e] = acc[e];
  __syncthreads();
  if (w == 0 && active) {
    Acc* dst = (Acc*)a.ws + (o * a.tiles_l + tl) * a.inner + col;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      Acc v = tot[0][lane * VEC + e];
#pragma unroll
      for (int ww = 1; ww < kScanWaves; ++ww) v += tot[ww][lane * VEC + e];
      dst[e] = v;
    }
  }
}

// pass B: ws[o][0..tiles_l)[col] -> exclusive prefix along the tile index, in place.  One 1024-lane workgroup per
// strip of 64 columns; wave w owns a contiguous range of tiles.
template <class Acc>
__global__ __launch_bounds__(kColBlock) void colscan_prefix_kernel(Acc* ws, int64_t tiles_l, int64_t inner, int64_t strips) {
  __shared__ Acc tot[kColWaves][kWave];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t strip = blockIdx.x % strips, o = blockIdx.x / strips;
  const int64_t col = strip * kWave + lane;
  const bool active = col < inner;
  Acc* p = ws + o * tiles_l * inner + (active ? col : 0);
  const int64_t per = (tiles_l + kColWaves - 1) / kColWaves;
  const int64_t t0 = w * per, t1 = t0 + per < tiles_l ? t0 + per : tiles_l;
  Acc sum = Acc(0);
  for (int64_t t = t0; t < t1; ++t) sum += p[t * inner];
  tot[w][lane] = sum;
  __syncthreads();
  Acc run = Acc(0);
  for (int ww = 0; ww < w; ++ww) run += tot[ww][lane];
  if (active) {
    for (int64_t t = t0; t < t1; ++t) {
      const Acc v = p[t * inner];
      p[t * inner] = run;
      run += v;
    }
  }
}

// pass C: scan the tile from registers, add the tile's prefix, write
template <class T, class O, class Acc, int VEC>
__global__ __launch_bounds__(kBlock) void colscan_apply_kernel(const ColArgs a) {
  __shared__ Acc tot[2][kScanWaves][kWave * VEC];
  int64_t o, tl, row0, row1, col;
  bool active;
  col_block<T, Acc, VEC>(a, &o, &tl, &row0, &row1, &col, &active);
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  int64_t xo, oo;
  slice_offsets(a.outer, o, &xo, &oo);
  const T* xp = (const T*)a.x + xo + (active ? col : 0);
  O* op = (O*)a.out + oo + (active ? col : 0);
  Acc carry[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) carry[e] = Acc(0);
  if (a.tiles_l > 1 && active) {
    const Acc* src = (const Acc*)a.ws + (o * a.tiles_l + tl) * a.inner + col;
#pragma unroll
    for (int e = 0; e < VEC; ++e) carry[e] = src[e];
  }
  int buf = 0;
  for (int64_t sub = row0; sub < row1; sub += kScanStep, buf ^= 1) {
    const int64_t rbase = sub + (int64_t)w * kScanRows;
    Vec<T, VEC> t[kScanRows];
#pragma unroll
    for (int r = 0; r < kScanRows; ++r) {
      const int64_t lr = rbase + r;
      t[r] = vec_load<T, VEC, true>(xp + (lr < row1 ? lr : row1 - 1) * a.xs);
    }
    Acc v[kScanRows][VEC];
#pragma unroll
    for (int r = 0; r < kScanRows; ++r) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const Acc xv = rbase + r < row1 ? cvt<Acc>(t[r].v[e]) : Acc(0);
        v[r][e] = r ? v[r - 1][e] + xv : xv;
      }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) tot[buf][w][lane * VEC + e] = v[kScanRows - 1][e];
    __syncthreads();                       // one barrier per step: the two LDS buffers alternate
    Acc off[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      Acc run = carry[e];
      off[e] = run;
#pragma unroll
      for (int ww = 0; ww < kScanWaves; ++ww) {
        if (ww == w) off[e] = run;
        run += tot[buf][ww][lane * VEC + e];
      }
      carry[e] = run;
    }
    if (active) {
#pragma unroll
      for (int r = 0; r < kScanRows; ++r) {
        if (rbase + r < row1) {
          Vec<O, VEC> res;
#pragma unroll
          for (int e = 0; e < VEC; ++e) res.v[e] = cvt<O>(v[r][e] + off[e]);
          vec_store<O, VEC, true>(op + (rbase + r) * a.os, res);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// host
// ---------------------------------------------------------------------------
struct ColLayout {
  int64_t L, inner, xs, os;
  Slices outer;
};

// dims after `dim` merge into one contiguous run in both tensors
bool cols_layout(const tx_tensor* out, const tx_tensor* x, int dim, ColLayout* c) {
  const int nd = x->ndim;
  if (nd < 2 || dim >= nd - 1) return false;
  int64_t inner = 1;
  for (int d = nd - 1; d > dim; --d) {
    if (x->sizes[d] != 1 && (x->strides[d] != inner || out->strides[d] != inner)) return false;
    inner *= x->sizes[d];
  }
  c->L = x->sizes[dim];
  c->inner = inner;
  c->xs = x->strides[dim];
  c->os = out->strides[dim];
  if (c->L < 2 || inner < 16) return false;
  build_slices_range(&c->outer, x, out, 0, dim, -1);
  return c->outer.count < (1ll << 31) && inner < (1ll << 40);
}

template <class T, class O> bool cols_aligned(const tx_tensor* out, const tx_tensor* x, const ColLayout& c, int vec) {
  if (vec == 1) return true;
  const int64_t xb = vec * (int64_t)sizeof(T), ob = vec * (int64_t)sizeof(O);
  bool al = c.inner % vec == 0 && (uintptr_t)x->data % xb == 0 && (uintptr_t)out->data % ob == 0 &&
            (c.xs * (int64_t)sizeof(T)) % xb == 0 && (c.os * (int64_t)sizeof(O)) % ob == 0;
  for (int d = 0; d < c.outer.n; ++d)
    al = al && (c.outer.xs[d] * (int64_t)sizeof(T)) % xb == 0 && (c.outer.os[d] * (int64_t)sizeof(O)) % ob == 0;
  return al;
}

void fill_args(ColArgs* a, const tx_tensor* out, const tx_tensor* x, const ColLayout& c, int cw) {
  memset(a, 0, sizeof(*a));
  a->x = (const char*)x->data;
  a->out = (char*)out->data;
  a->outer = c.outer;
  a->L = c.L;
  a->inner = c.inner;
  a->xs = c.xs;
  a->os = c.os;
  a->col_tiles = (c.inner + cw - 1) / cw;
}

template <class T, class O>
tx_status softmax_cols_typed(const tx_tensor* out, const tx_tensor* x, const ColLayout& c, int is_log, hipStream_t stream) {
  constexpr int V = sizeof(T) == 2 ? 4 : 16 / sizeof(T);    // 4 columns per lane
  ColArgs a;
  // widest strip that still gives the chip enough workgroups
  const bool al = cols_aligned<T, O>(out, x, c, V);
  int cw = al ? kWave * V : kWave;
  if (al && c.outer.count * ((c.inner + cw - 1) / cw) < 512) cw = kWave;
  const bool narrow = c.outer.count * ((c.inner + kWave - 1) / kWave) < 512 && cw == kWave;
  if (narrow) cw = 16;
  fill_args(&a, out, x, c, cw);
  a.is_log = is_log;
  const int64_t blocks = c.outer.count * a.col_tiles;
  if (blocks >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "softmax: too many column strips");
  set_path("softmax-cols");
  const dim3 grid((unsigned)blocks);
  if (cw == kWave * V) hipLaunchKernelGGL((softmax_cols_kernel<T, O, V, kWave>), grid, dim3(kColBlock), 0, stream, a);
  else if (cw == kWave) hipLaunchKernelGGL((softmax_cols_kernel<T, O, 1, kWave>), grid, dim3(kColBlock), 0, stream, a);
  else hipLaunchKernelGGL((softmax_cols_kernel<T, O, 1, 16>), grid, dim3(kColBlock), 0, stream, a);
  return check_launch("softmax column kernel");
}

template <class T, class O, class Acc>
tx_status cumsum_cols_typed(const tx_tensor* out, const tx_tensor* x, const ColLayout& c, void* ws, size_t ws_bytes,
                            hipStream_t stream, size_t* query) {
  constexpr int V0 = sizeof(T) >= 8 ? 2 : 4;
  const bool al = cols_aligned<T, O>(out, x, c, V0);
  const int V = al ? V0 : 1;
  ColArgs a;
  fill_args(&a, out, x, c, kWave * V);
  // rows per workgroup: a multiple of the step, few enough tiles that the chip still gets ~2048 workgroups
  const int64_t strips = c.outer.count * a.col_tiles;
  const int64_t want_tiles = std::max<int64_t>(1, (2048 + strips - 1) / strips);
  int64_t rpb = (c.L + want_tiles - 1) / want_tiles;
  rpb = std::max<int64_t>(kScanStep, (rpb + kScanStep - 1) / kScanStep * kScanStep);
  a.rows_per_block = rpb;
  a.tiles_l = (c.L + rpb - 1) / rpb;
  const size_t need = a.tiles_l > 1 ? (size_t)c.outer.count * a.tiles_l * c.inner * sizeof(Acc) : 0;
  if (query) { *query = need; return TX_OK; }
  const int64_t blocks = strips * a.tiles_l;
  if (blocks >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "cumsum: too many tiles");
  if (need && (!ws || ws_bytes < need)) return fail(TX_ERR_WORKSPACE, "cumsum needs %zu workspace bytes, got %zu", need, ws_bytes);
  if (need && (uintptr_t)ws % 8) return fail(TX_ERR_WORKSPACE, "cumsum workspace must be 8-byte aligned");
  a.ws = (char*)ws;
  const dim3 grid((unsigned)blocks);
  if (a.tiles_l > 1) {
    if (V > 1) hipLaunchKernelGGL((colscan_sums_kernel<T, Acc, V0>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((colscan_sums_kernel<T, Acc, 1>), grid, dim3(kBlock), 0, stream, a);
    const int64_t pstrips = (c.inner + kWave - 1) / kWave;
    hipLaunchKernelGGL((colscan_prefix_kernel<Acc>), dim3((unsigned)(c.outer.count * pstrips)), dim3(kColBlock), 0, stream,
                       (Acc*)ws, a.tiles_l, c.inner, pstrips);
  }
  set_path(V > 1 ? "scan-cols" : "scan-cols-scalar");
  if (V > 1) hipLaunchKernelGGL((colscan_apply_kernel<T, O, Acc, V0>), grid, dim3(kBlock), 0, stream, a);
  else hipLaunchKernelGGL((colscan_apply_kernel<T, O, Acc, 1>), grid, dim3(kBlock), 0, stream, a);
  return check_launch("cumsum column kernels");
}

}  // namespace

bool cols_path_ok(const tx_tensor* out, const tx_tensor* x, int dim) {
  ColLayout c;
  return cols_layout(out, x, dim, &c);
}

tx_status softmax_cols(const tx_tensor* out, const tx_tensor* x, int dim, int is_log, hipStream_t stream) {
  ColLayout c;
  if (!cols_layout(out, x, dim, &c)) return fail(TX_ERR_UNSUPPORTED, "softmax: not a column layout");
  const bool wide = out->dtype == TX_F32;
  switch (x->dtype) {
    case TX_F32: return softmax_cols_typed<float, float>(out, x, c, is_log, stream);
    case TX_BF16: return wide ? softmax_cols_typed<bf16, float>(out, x, c, is_log, stream) : softmax_cols_typed<bf16, bf16>(out, x, c, is_log, stream);
    default: return wide ? softmax_cols_typed<f16, float>(out, x, c, is_log, stream) : softmax_cols_typed<f16, f16>(out, x, c, is_log, stream);
  }
}

tx_status cumsum_cols(const tx_tensor* out, const tx_tensor* x, int dim, void* ws, size_t wsb, hipStream_t s, size_t* query) {
  ColLayout c;
  if (!cols_layout(out, x, dim, &c)) return fail(TX_ERR_UNSUPPORTED, "cumsum: not a column layout");
  const bool wide = out->dtype == TX_F32;
  switch (x->dtype) {
    case TX_BOOL: return cumsum_cols_typed<uint8_t, int64_t, int64_t>(out, x, c, ws, wsb, s, query);
    case TX_I32: return cumsum_cols_typed<int32_t, int64_t, int64_t>(out, x, c, ws, wsb, s, query);
    case TX_I64: return cumsum_cols_typed<int64_t, int64_t, int64_t>(out, x, c, ws, wsb, s, query);
    case TX_F32: return cumsum_cols_typed<float, float, float>(out, x, c, ws, wsb, s, query);
    case TX_BF16:
      return wide ? cumsum_cols_typed<bf16, float, float>(out, x, c, ws, wsb, s, query)
                  : cumsum_cols_typed<bf16, bf16, float>(out, x, c, ws, wsb, s, query);
    default:
      return wide ? cumsum_cols_typed<f16, float, float>(out, x, c, ws, wsb, s, query)
                  : cumsum_cols_typed<f16, f16, float>(out, x, c, ws, wsb, s, query);
  }
}

}  // namespace tx
