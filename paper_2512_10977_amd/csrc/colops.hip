// softmax / log_softmax and cumsum along a dim that is NOT the innermost one,
// for tensors whose dims after it form one contiguous run ("columns"): the
// tensor is seen as [outer..., L, inner] with inner contiguous.  Lanes run
// along `inner` (coalesced), the operated dim is walked with its stride.
//
// softmax : a 1024-lane workgroup owns a strip of columns; its 16 waves take
//           interleaved rows and keep a running (max, scaled sum) per column,
//           merge through LDS, then read the strip again and write.  Two
//           reads and one write per element.  An operated dim of at most 128
//           stays in registers instead: one read.
// cumsum  : the rows are cut into tiles.  Pass A sums every tile per column
//           into the workspace, pass B turns those sums into exclusive
//           prefixes (in place), pass C scans every tile from registers,
//           adds its prefix and writes.  Two reads and one write per element;
//           with a single tile per column passes A and B are skipped.
//           Columns too long for one tile take a single-pass form instead:
//           tiles of 128 rows, drawn by ticket, whose column totals travel
//           between workgroups by decoupled look-back (one read, one write).
#include <cstring>

#include "common.h"
#include "rows.h"
#include "scan_impl.h"

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
  constexpr int RL = kWave / CPW, CW = CPW * VEC, RS = kColWaves * RL, U = VEC == 1 ? 16 : 4;
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

// The same for a short operated dim (L <= 128): the strip's L rows stay in registers - wave w of NW holds rows
// 16 w .. 16 w + 15, lane l the columns VEC l .. - so the input is read once.  The arithmetic is that of the row
// kernels: column maximum, exp(x - m) summed in row order per wave and then in wave order, one division per column.
// Workgroups are as small as L allows (64 to 512 lanes), so that several are resident per CU and one's loads overlap
// another's stores.
constexpr int kCRRows = 16;
template <class T, class O, int VEC, int NW>
__global__ __launch_bounds__(NW * kWave) void softmax_cols_reg_kernel(const ColArgs a) {
  constexpr int CW = kWave * VEC;
  __shared__ float lm[NW][CW], ls[NW][CW];
  const int lane = threadIdx.x & (kWave - 1);
  const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int64_t tile = blockIdx.x % a.col_tiles, o = blockIdx.x / a.col_tiles;
  int64_t xo, oo;
  slice_offsets(a.outer, o, &xo, &oo);
  const int64_t col = tile * CW + (int64_t)lane * VEC;
  const bool active = col < a.inner;                       // inner is a multiple of VEC when VEC > 1
  const T* xp = (const T*)a.x + xo + (active ? col : 0);
  O* op = (O*)a.out + oo + (active ? col : 0);
  const int64_t rbase = (int64_t)w * kCRRows;
  const int c0 = lane * VEC;
  Vec<T, VEC> t[kCRRows];
#pragma unroll
  for (int r = 0; r < kCRRows; ++r) {
    const int64_t lr = rbase + r;
    t[r] = vec_load<T, VEC, true>(xp + (lr < a.L ? lr : a.L - 1) * a.xs);
  }
  float v[kCRRows][VEC], m[VEC], s[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) m[e] = kNegInf;
#pragma unroll
  for (int r = 0; r < kCRRows; ++r) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      v[r][e] = rbase + r < a.L ? cvt<float>(t[r].v[e]) : kNegInf;
      m[e] = fmaxf(m[e], v[r][e]);
    }
  }
  if constexpr (NW > 1) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) lm[w][c0 + e] = m[e];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      float M = lm[0][c0 + e];
#pragma unroll
      for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, lm[ww][c0 + e]);
      m[e] = M;
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) s[e] = 0.0f;
#pragma unroll
  for (int r = 0; r < kCRRows; ++r) {
    if (rbase + r < a.L) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float d = v[r][e] - m[e];
        const float ex = expf(d);
        s[e] += ex;
        v[r][e] = a.is_log ? d : ex;
      }
    }
  }
  if constexpr (NW > 1) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) ls[w][c0 + e] = s[e];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      float S = ls[0][c0 + e];
#pragma unroll
      for (int ww = 1; ww < NW; ++ww) S += ls[ww][c0 + e];
      s[e] = S;
    }
  }
  float inv[VEC], lg[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    inv[e] = 1.0f / s[e];
    lg[e] = logf(s[e]);
  }
  if (active) {
#pragma unroll
    for (int r = 0; r < kCRRows; ++r) {
      if (rbase + r < a.L) {
        Vec<O, VEC> res;
#pragma unroll
        for (int e = 0; e < VEC; ++e) res.v[e] = cvt<O>(a.is_log ? v[r][e] - lg[e] : v[r][e] * inv[e]);
        vec_store<O, VEC, true>(op + (rbase + r) * a.os, res);
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
// cumsum along columns in one pass: decoupled look-back between row tiles
// ---------------------------------------------------------------------------
// A workgroup of 8 waves owns a tile of 128 rows x (64 VEC) columns: wave w holds rows 16 w .. 16 w + 15 of the tile in
// registers, lane l the columns VEC l .. VEC l + VEC - 1.  The tile's column totals are published as AGGREGATE status
// words (one flagged word per column, the layout of the row scan's tile status), the exclusive prefix of every column
// is collected from the tiles above it, and the inclusive prefix is published for the tiles below.  Tiles are drawn by
// ticket, all strips of one tile row before the next tile row, so a tile's predecessors always hold earlier tickets
// (they are running or done, and publish their aggregate without waiting on anyone).  Each look-back round inspects
// 8 predecessors at once, one per wave: the waves park what they read in LDS, and every wave then folds the 8 entries
// nearest-first for its own columns until it meets an inclusive prefix (all waves reach the same verdict from the same
// LDS data, so the loop's exit is uniform without a vote).  Every wait is bounded like the row scan's.
// Measured on [4096,32768] / [65536,2048] fp32 (196 / 227 us; the three-pass form 271 / 290 us): tiles of 64 rows
// 219 / 310 us (twice the tickets and look-backs per byte), 16 predecessors per round 205 / 244 us, a persistent grid
// of two workgroups per CU that draws the next ticket ahead 201 / 285 us.
constexpr int kCLWaves = 8;
constexpr int kCLBlock = kCLWaves * kWave;
constexpr int kCLRows = 16;                            // rows per wave
constexpr int kCLTileRows = kCLWaves * kCLRows;        // 128
constexpr int kCLLook = kCLWaves;                      // predecessors inspected per look-back round

struct ColLookArgs {
  const char* x;
  char* out;
  char* ws;
  Slices outer;
  int64_t L, inner, xs, os;
  int64_t col_tiles;            // column strips per outer slice
  int64_t strips;               // outer slices x col_tiles
  int64_t tiles_l, total_tiles;
  int spin_limit;
};

template <class T, class O, class Acc, int VEC>
__global__ __launch_bounds__(kCLBlock) void colscan_lookback_kernel(const ColLookArgs a) {
  constexpr int CW = kWave * VEC;
  __shared__ Acc tot[kCLWaves][CW];
  __shared__ Acc lbv[2][kCLLook][CW];
  __shared__ uint8_t lbf[2][kCLLook][CW];
  __shared__ unsigned int my_ticket;
  ScanHeader* hdr = (ScanHeader*)a.ws;
  unsigned long long* status = (unsigned long long*)(a.ws + 256);
  if (threadIdx.x == 0) my_ticket = atomicAdd(&hdr->ticket, 1u);
  __syncthreads();
  const int64_t ticket = my_ticket;
  if (ticket >= a.total_tiles) return;
  const int64_t tl = ticket / a.strips, sg = ticket - tl * a.strips;
  const int64_t o = sg / a.col_tiles, strip = sg - o * a.col_tiles;
  const int lane = threadIdx.x & (kWave - 1);
  const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  int64_t xo, oo;
  slice_offsets(a.outer, o, &xo, &oo);
  const int64_t col = strip * CW + (int64_t)lane * VEC;
  const bool active = col < a.inner;                       // inner is a multiple of VEC when VEC > 1
  const T* xp = (const T*)a.x + xo + (active ? col : 0);
  O* op = (O*)a.out + oo + (active ? col : 0);
  const int64_t rbase = tl * kCLTileRows + (int64_t)w * kCLRows;
  const int c0 = lane * VEC;

  Vec<T, VEC> t[kCLRows];
#pragma unroll
  for (int r = 0; r < kCLRows; ++r) {
    const int64_t lr = rbase + r;
    t[r] = vec_load<T, VEC, true>(xp + (lr < a.L ? lr : a.L - 1) * a.xs);
  }
  Acc v[kCLRows][VEC];
#pragma unroll
  for (int r = 0; r < kCLRows; ++r) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const Acc xv = rbase + r < a.L ? cvt<Acc>(t[r].v[e]) : Acc(0);
      v[r][e] = r ? v[r - 1][e] + xv : xv;
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) tot[w][c0 + e] = v[kCLRows - 1][e];
  __syncthreads();
  Acc woff[VEC], agg[VEC], prefix[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    Acc run = Acc(0);
    woff[e] = run;
#pragma unroll
    for (int ww = 0; ww < kCLWaves; ++ww) {
      if (ww == w) woff[e] = run;
      run += tot[ww][c0 + e];
    }
    agg[e] = run;
    prefix[e] = Acc(0);
  }
  const int64_t slot0 = sg * a.tiles_l;                    // status slots of this strip, one per tile row
  if (tl > 0) {
    if (w == 0 && active) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) TileState<Acc>::publish(status, (slot0 + tl) * CW + c0 + e, kAggregate, agg[e]);
    }
    bool done[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) done[e] = !active;
    int buf = 0;
    for (int64_t look = tl - 1;; look -= kCLLook, buf ^= 1) {
#pragma unroll
      for (int j = 0; j < kCLLook / kCLWaves; ++j) {
        const int slot = j * kCLWaves + w;                 // wave w inspects tile row look - w (uniform per wave)
        const int64_t mine = look - slot;
        Acc val[VEC];
        uint32_t flag[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          val[e] = Acc(0);
          flag[e] = kPrefix;                               // rows above the tensor count as an empty prefix
        }
        if (mine >= 0) {
          // the status words of a lane's columns are requested together; a column that is through reads nothing
          bool ready = false;
          for (int spins = 0; spins < a.spin_limit && !ready; ++spins) {      // a limit of 0 (host-forced, for tests) gives up at once
            ready = true;
#pragma unroll
            for (int e = 0; e < VEC; ++e)
              if (!done[e]) flag[e] = TileState<Acc>::read(status, (slot0 + mine) * CW + c0 + e, &val[e]);
#pragma unroll
            for (int e = 0; e < VEC; ++e) ready = ready && flag[e] != kEmpty;
            if (!ready) __builtin_amdgcn_s_sleep(2);
          }
          if (!ready) {
#pragma unroll
            for (int e = 0; e < VEC; ++e)
              if (!done[e] && (a.spin_limit == 0 || flag[e] == kEmpty)) { hdr->error = 1; flag[e] = kPrefix; val[e] = Acc(0); }
          }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          lbv[buf][slot][c0 + e] = val[e];
          lbf[buf][slot][c0 + e] = (uint8_t)flag[e];
        }
      }
      __syncthreads();                                     // one barrier per round: the two LDS buffers alternate
      bool all = true;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
#pragma unroll
        for (int ww = 0; ww < kCLLook; ++ww) {
          if (!done[e]) {
            prefix[e] = lbv[buf][ww][c0 + e] + prefix[e];
            done[e] = lbf[buf][ww][c0 + e] == (uint8_t)kPrefix;
          }
        }
        all = all && done[e];
      }
      if (__ballot(!all) == 0ull) break;
    }
  }
  if (w == 0 && active) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) TileState<Acc>::publish(status, (slot0 + tl) * CW + c0 + e, kPrefix, (Acc)(prefix[e] + agg[e]));
  }
  if (active) {
#pragma unroll
    for (int r = 0; r < kCLRows; ++r) {
      if (rbase + r < a.L) {
        Vec<O, VEC> res;
#pragma unroll
        for (int e = 0; e < VEC; ++e) res.v[e] = cvt<O>((Acc)(v[r][e] + (prefix[e] + woff[e])));
        vec_store<O, VEC, true>(op + (rbase + r) * a.os, res);
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
  const bool al = cols_aligned<T, O>(out, x, c, V);
  // a short operated dim stays in registers: one read of the input ("softmax-cols" by name keeps the two-read form)
  if (c.L <= 8 * kCRRows && strcmp(forced_path(), "softmax-cols") != 0) {
    fill_args(&a, out, x, c, al ? kWave * V : kWave);
    a.is_log = is_log;
    const int64_t nb = c.outer.count * a.col_tiles;
    if (nb >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "softmax: too many column strips");
    set_path(al ? "softmax-cols-reg" : "softmax-cols-reg-scalar");
    const dim3 g((unsigned)nb);
    const int nw = c.L <= kCRRows ? 1 : c.L <= 2 * kCRRows ? 2 : c.L <= 4 * kCRRows ? 4 : 8;
#define TX_COLS_REG(VV)                                                                                                   \
    switch (nw) {                                                                                                         \
      case 1: hipLaunchKernelGGL((softmax_cols_reg_kernel<T, O, VV, 1>), g, dim3(kWave), 0, stream, a); break;           \
      case 2: hipLaunchKernelGGL((softmax_cols_reg_kernel<T, O, VV, 2>), g, dim3(2 * kWave), 0, stream, a); break;       \
      case 4: hipLaunchKernelGGL((softmax_cols_reg_kernel<T, O, VV, 4>), g, dim3(4 * kWave), 0, stream, a); break;       \
      default: hipLaunchKernelGGL((softmax_cols_reg_kernel<T, O, VV, 8>), g, dim3(8 * kWave), 0, stream, a); break;      \
    }
    if (al) { TX_COLS_REG(V) } else { TX_COLS_REG(1) }
#undef TX_COLS_REG
    return check_launch("softmax column kernel (registers)");
  }
  // widest strip that still gives the chip enough workgroups
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
  // a 64-column strip of an aligned tensor: 16 column-lanes of 4 columns, so that a wave's load still moves 1 KiB
  // (four row segments of 256 bytes) and a lane holds 64 bytes in flight instead of 16
  else if (cw == kWave && al) hipLaunchKernelGGL((softmax_cols_kernel<T, O, V, kWave / V>), grid, dim3(kColBlock), 0, stream, a);
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
  const size_t need3 = a.tiles_l > 1 ? (size_t)c.outer.count * a.tiles_l * c.inner * sizeof(Acc) : 0;
  // columns cut into several tiles: the single-pass look-back form, unless the three-pass one is asked for by name.
  // The workspace query answers for both, so that a forced path never finds the workspace short.
  // (8-byte accumulators take two columns per lane there: 16 rows x 4 columns of them would leave one workgroup per CU)
  constexpr int VL0 = sizeof(Acc) >= 8 ? 2 : V0;
  const int VL = al ? VL0 : 1;
  const int64_t look_col_tiles = (c.inner + kWave * VL - 1) / (kWave * VL);
  const int64_t look_strips = c.outer.count * look_col_tiles;
  const int64_t look_tiles_l = (c.L + kCLTileRows - 1) / kCLTileRows;
  const int64_t look_total = look_strips * look_tiles_l;
  const size_t need_look = a.tiles_l > 1 ? 256 + (size_t)look_total * (kWave * VL) * TileState<Acc>::words * 8 : 0;
  const size_t need = std::max(need3, need_look);
  if (query) { *query = need; return TX_OK; }
  const int64_t blocks = strips * a.tiles_l;
  if (blocks >= (1ll << 31) || look_total >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "cumsum: too many tiles");
  if (need && (!ws || ws_bytes < need)) return fail(TX_ERR_WORKSPACE, "cumsum needs %zu workspace bytes, got %zu", need, ws_bytes);
  if (need && (uintptr_t)ws % 8) return fail(TX_ERR_WORKSPACE, "cumsum workspace must be 8-byte aligned");
  a.ws = (char*)ws;
  const bool giveup = !strcmp(forced_path(), "scan-cols-lookback-giveup");
  if (a.tiles_l > 1 && strcmp(forced_path(), "scan-cols-3pass") != 0) {
    ColLookArgs k;
    memset(&k, 0, sizeof(k));
    k.x = a.x;
    k.out = a.out;
    k.ws = (char*)ws;
    k.outer = c.outer;
    k.L = c.L;
    k.inner = c.inner;
    k.xs = c.xs;
    k.os = c.os;
    k.col_tiles = look_col_tiles;
    k.strips = look_strips;
    k.tiles_l = look_tiles_l;
    k.total_tiles = look_total;
    k.spin_limit = giveup ? 0 : kSpinLimit;
    const int64_t words = (int64_t)(need_look / 8);
    hipLaunchKernelGGL(scan_clear_kernel, dim3((unsigned)((words + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream,
                       (unsigned long long*)ws, words);
    set_path(VL > 1 ? "scan-cols-lookback" : "scan-cols-lookback-scalar");
    const dim3 lgrid((unsigned)look_total);
    if (VL > 1) hipLaunchKernelGGL((colscan_lookback_kernel<T, O, Acc, VL0>), lgrid, dim3(kCLBlock), 0, stream, k);
    else hipLaunchKernelGGL((colscan_lookback_kernel<T, O, Acc, 1>), lgrid, dim3(kCLBlock), 0, stream, k);
    return check_launch("cumsum column look-back kernel");
  }
  const dim3 grid((unsigned)blocks);
  if (a.tiles_l > 1) {
    if (V > 1) hipLaunchKernelGGL((colscan_sums_kernel<T, Acc, V0>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((colscan_sums_kernel<T, Acc, 1>), grid, dim3(kBlock), 0, stream, a);
    const int64_t pstrips = (c.inner + kWave - 1) / kWave;
    hipLaunchKernelGGL((colscan_prefix_kernel<Acc>), dim3((unsigned)(c.outer.count * pstrips)), dim3(kColBlock), 0, stream,
                       (Acc*)ws, a.tiles_l, c.inner, pstrips);
  }
  set_path(V > 1 ? (a.tiles_l > 1 ? "scan-cols-3pass" : "scan-cols") : (a.tiles_l > 1 ? "scan-cols-3pass-scalar" : "scan-cols-scalar"));
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
