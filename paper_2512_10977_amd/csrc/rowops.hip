// Row operators: softmax / log_softmax and cumsum along one dim.
//
// softmax, last dim contiguous:
//   wave  : one wave64 owns a row and keeps it in registers (up to 1024
//           16-byte vectors, i.e. 4096 fp32 or 8192 half elements): one HBM
//           read, two wave reductions (max, sum), one HBM write.
//   block : longer rows; a 256-lane workgroup makes three passes over the row
//           (the re-reads are served by L2).
// softmax / cumsum along another dim whose trailing dims are contiguous: the column kernels of colops.hip.
// Anything else (strided slices, short trailing runs):
//   strided: one lane per slice, walking the dim with its stride (lanes run
//           along the innermost other dim, so accesses stay coalesced when
//           that dim is contiguous).
// cumsum, last dim contiguous: single-pass scan with decoupled look-back.  A
//   row is cut into tiles; a workgroup takes tiles in ticket order, scans its
//   tile, publishes the tile aggregate, and resolves its exclusive prefix by
//   looking back over predecessor tiles' published aggregates / inclusive
//   prefixes.  Each element is read once and written once.
#include <algorithm>
#include <cstring>

#include "common.h"
#include "rows.h"

namespace tx {
namespace {

template <class O> __device__ __forceinline__ O from_float(float v) { return cvt<O>(v); }

// ---------------------------------------------------------------------------
// softmax
// ---------------------------------------------------------------------------
struct SoftmaxArgs {
  const char* x;
  char* out;
  int64_t rows, len;
  int64_t xrow, orow;     // row strides in elements
  int is_log;
};

// one wave per row, CH vectors of VEC elements per lane
template <class T, class O, int VEC, int CH>
__global__ __launch_bounds__(kBlock) void softmax_wave_kernel(const SoftmaxArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t row = (int64_t)blockIdx.x * (kBlock / kWave) + (threadIdx.x / kWave);
  if (row >= a.rows) return;
  const T* x = (const T*)a.x + row * a.xrow;
  O* out = (O*)a.out + row * a.orow;
  float v[CH][VEC];
  float m = kNegInf;
  // Loads go out in groups of up to 8, every one of them unconditional (a vector past the end of the row
  // re-reads the row's first vector and is replaced by -inf afterwards): a load inside `if (c < len)` is
  // waited for inside that branch, which leaves one load in flight per wave.
  constexpr int kGroup = CH < 8 ? CH : 8;
#pragma unroll
  for (int k0 = 0; k0 < CH; k0 += kGroup) {
    Vec<T, VEC> t[kGroup];
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
      const int64_t c = ((int64_t)(k0 + j) * kWave + lane) * VEC;
      t[j] = vec_load<T, VEC, true>(x + (c < a.len ? c : 0));      // len is a multiple of VEC on this path
    }
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
      const int64_t c = ((int64_t)(k0 + j) * kWave + lane) * VEC;
      const bool in = c < a.len;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        v[k0 + j][e] = in ? cvt<float>(t[j].v[e]) : kNegInf;
        m = fmaxf(m, v[k0 + j][e]);
      }
    }
  }
  m = wave_max(m);
  float s = 0.0f;
#pragma unroll
  for (int k = 0; k < CH; ++k) {
    const int64_t c = ((int64_t)k * kWave + lane) * VEC;
    if (c < a.len) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        v[k][e] -= m;
        const float ex = expf(v[k][e]);
        s += ex;
        if (!a.is_log) v[k][e] = ex;
      }
    }
  }
  s = wave_sum(s);
  const float inv = 1.0f / s, ls = logf(s);
#pragma unroll
  for (int k = 0; k < CH; ++k) {
    const int64_t c = ((int64_t)k * kWave + lane) * VEC;
    if (c < a.len) {
      Vec<O, VEC> t;
#pragma unroll
      for (int e = 0; e < VEC; ++e) t.v[e] = from_float<O>(a.is_log ? v[k][e] - ls : v[k][e] * inv);
      vec_store<O, VEC, true>(out + c, t);
    }
  }
}

// one workgroup per row, three passes
template <class T, class O>
__global__ __launch_bounds__(kBlock) void softmax_block_kernel(const SoftmaxArgs a) {
  __shared__ float lds[kBlock / kWave];
  const int64_t row = blockIdx.x;
  const T* x = (const T*)a.x + row * a.xrow;
  O* out = (O*)a.out + row * a.orow;
  float m = kNegInf;
  for (int64_t c = threadIdx.x; c < a.len; c += kBlock) m = fmaxf(m, cvt<float>(x[c]));
  m = block_reduce(m, true, lds);
  float s = 0.0f;
  for (int64_t c = threadIdx.x; c < a.len; c += kBlock) s += expf(cvt<float>(x[c]) - m);
  s = block_reduce(s, false, lds);
  const float inv = 1.0f / s, ls = logf(s);
  for (int64_t c = threadIdx.x; c < a.len; c += kBlock) {
    const float d = cvt<float>(x[c]) - m;
    out[c] = from_float<O>(a.is_log ? d - ls : expf(d) * inv);
  }
}

struct StridedArgs {
  const char* x;
  char* out;
  Slices sl;
  int64_t len, xs, os;    // extent and strides of the operated dim
  int is_log;
};

template <class T, class O>
__global__ __launch_bounds__(kBlock) void softmax_strided_kernel(const StridedArgs a) {
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (idx >= a.sl.count) return;
  int64_t xo, oo;
  slice_offsets(a.sl, idx, &xo, &oo);
  const T* x = (const T*)a.x + xo;
  O* out = (O*)a.out + oo;
  float m = kNegInf;
  for (int64_t j = 0; j < a.len; ++j) m = fmaxf(m, cvt<float>(x[j * a.xs]));
  float s = 0.0f;
  for (int64_t j = 0; j < a.len; ++j) s += expf(cvt<float>(x[j * a.xs]) - m);
  const float inv = 1.0f / s, ls = logf(s);
  for (int64_t j = 0; j < a.len; ++j) {
    const float d = cvt<float>(x[j * a.xs]) - m;
    out[j * a.os] = from_float<O>(a.is_log ? d - ls : expf(d) * inv);
  }
}

template <class T, class O>
tx_status softmax_launch(const tx_tensor* out, const tx_tensor* x, int dim, int is_log, hipStream_t stream) {
  constexpr int V = 16 / sizeof(T);
  const int nd = x->ndim;
  const int64_t len = nd ? x->sizes[dim] : 1;
  const int64_t xs = nd ? x->strides[dim] : 1, os = nd ? out->strides[dim] : 1;
  Slices sl;
  build_slices(&sl, x, out, nd ? dim : -1);
  if (sl.count >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "softmax: too many slices");
  const bool rows = (len == 1 || (xs == 1 && os == 1)) && sl.n <= 1 && len > 1;
  if (rows) {
    SoftmaxArgs a;
    a.x = (const char*)x->data;
    a.out = (char*)out->data;
    a.rows = sl.count;
    a.len = len;
    a.xrow = sl.n ? sl.xs[0] : 0;
    a.orow = sl.n ? sl.os[0] : 0;
    a.is_log = is_log;
    const bool al = len % V == 0 && (uintptr_t)x->data % 16 == 0 && (uintptr_t)out->data % (V * sizeof(O) >= 16 ? 16 : V * sizeof(O)) == 0 &&
                    (a.xrow * (int64_t)sizeof(T)) % 16 == 0 && (a.orow * (int64_t)sizeof(O)) % 16 == 0;
    const dim3 grid((unsigned)((a.rows + 3) / 4));
    if (al && len <= 64 * V) {
      set_path("softmax-wave");
      hipLaunchKernelGGL((softmax_wave_kernel<T, O, V, 1>), grid, dim3(kBlock), 0, stream, a);
    } else if (al && len <= 256 * V) {
      set_path("softmax-wave");
      hipLaunchKernelGGL((softmax_wave_kernel<T, O, V, 4>), grid, dim3(kBlock), 0, stream, a);
    } else if (al && len <= 512 * V) {
      set_path("softmax-wave");
      hipLaunchKernelGGL((softmax_wave_kernel<T, O, V, 8>), grid, dim3(kBlock), 0, stream, a);
    } else if (al && len <= 1024 * V) {
      set_path("softmax-wave");
      hipLaunchKernelGGL((softmax_wave_kernel<T, O, V, 16>), grid, dim3(kBlock), 0, stream, a);
    } else if (len <= 64 * 16) {
      set_path("softmax-wave-scalar");
      hipLaunchKernelGGL((softmax_wave_kernel<T, O, 1, 16>), grid, dim3(kBlock), 0, stream, a);
    } else {
      set_path("softmax-block");
      hipLaunchKernelGGL((softmax_block_kernel<T, O>), dim3((unsigned)a.rows), dim3(kBlock), 0, stream, a);
    }
    return check_launch("softmax kernel");
  }
  if (nd && strcmp(forced_path(), "softmax-strided") && cols_path_ok(out, x, dim)) return softmax_cols(out, x, dim, is_log, stream);
  StridedArgs a;
  a.x = (const char*)x->data;
  a.out = (char*)out->data;
  a.sl = sl;
  a.len = len;
  a.xs = xs;
  a.os = os;
  a.is_log = is_log;
  set_path("softmax-strided");
  hipLaunchKernelGGL((softmax_strided_kernel<T, O>), dim3((unsigned)((sl.count + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                     stream, a);
  return check_launch("softmax strided kernel");
}

// ---------------------------------------------------------------------------
// cumsum: decoupled look-back scan
// ---------------------------------------------------------------------------
constexpr int kNV = 4;                       // vectors per lane per tile
constexpr uint32_t kEmpty = 0, kAggregate = 1, kPrefix = 2;
constexpr int kSpinLimit = 1 << 24;          // bounded wait: a stuck predecessor sets the error word instead of hanging

struct ScanHeader {                           // first 256 bytes of the workspace
  unsigned int ticket;
  unsigned int error;
};

// Tile status.  4-byte accumulators travel with their flag in one 64-bit word.
// 8-byte accumulators use two flagged words per value, and separate slots for
// the aggregate and the inclusive prefix so that every word is written once.
template <class Acc> struct TileState;
template <> struct TileState<float> {
  static constexpr int words = 1;
  __device__ static void publish(unsigned long long* st, int64_t tile, uint32_t flag, float v) {
    unsigned long long w = ((unsigned long long)flag << 32) | __float_as_uint(v);
    __hip_atomic_store(st + tile, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __device__ static uint32_t read(unsigned long long* st, int64_t tile, float* v) {
    unsigned long long w = __hip_atomic_load(st + tile, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *v = __uint_as_float((uint32_t)w);
    return (uint32_t)(w >> 32);
  }
};
template <> struct TileState<int64_t> {
  static constexpr int words = 4;
  __device__ static void publish(unsigned long long* st, int64_t tile, uint32_t flag, int64_t v) {
    unsigned long long* p = st + tile * 4 + (flag == kPrefix ? 2 : 0);
    const unsigned long long f = 1ull << 32;
    __hip_atomic_store(p, f | (uint32_t)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 1, f | (uint32_t)((unsigned long long)v >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __device__ static uint32_t read(unsigned long long* st, int64_t tile, int64_t* v) {
    unsigned long long* p = st + tile * 4;
    unsigned long long lo = __hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long hi = __hip_atomic_load(p + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((lo >> 32) && (hi >> 32)) { *v = (int64_t)((hi << 32) | (uint32_t)lo); return kPrefix; }
    lo = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    hi = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((lo >> 32) && (hi >> 32)) { *v = (int64_t)((hi << 32) | (uint32_t)lo); return kAggregate; }
    *v = 0;
    return kEmpty;
  }
};

__global__ void scan_clear_kernel(unsigned long long* ws, int64_t words) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < words) ws[i] = 0ull;
}

struct ScanArgs {
  const char* x;
  char* out;
  char* ws;
  int64_t rows, len, xrow, orow;
  int64_t tiles_per_row, total_tiles;
};

template <class Acc> __device__ __forceinline__ Acc wave_inclusive(Acc v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    Acc o = shfl_up(v, d);
    if (lane >= d) v += o;
  }
  return v;
}

// Loads one tile (NV vectors per lane, lanes interleaved) into accumulators.  A tile that lies wholly inside the
// row takes the first branch (uniform for the workgroup): NV unconditional vector loads, all in flight before
// the first conversion.  Only a ragged last tile takes the element-wise branch.
template <class T, class Acc, int VEC, int THREADS, int NV>
__device__ __forceinline__ void scan_tile_load_full(const T* xt, Acc (&dst)[NV][VEC]) {
  Vec<T, VEC> raw[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) raw[k] = vec_load<T, VEC, true>(xt + ((int64_t)k * THREADS + threadIdx.x) * VEC);
#pragma unroll
  for (int k = 0; k < NV; ++k)
#pragma unroll
    for (int e = 0; e < VEC; ++e) dst[k][e] = cvt<Acc>(raw[k].v[e]);
}
template <class T, class Acc, int VEC, int THREADS, int NV>
__device__ __forceinline__ void scan_tile_load(const T* xt, int64_t left, Acc (&dst)[NV][VEC]) {
  if (left >= (int64_t)THREADS * NV * VEC) {
    scan_tile_load_full<T, Acc, VEC, THREADS, NV>(xt, dst);
  } else {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int64_t c = ((int64_t)k * THREADS + threadIdx.x) * VEC;
#pragma unroll
      for (int e = 0; e < VEC; ++e) dst[k][e] = (c + e < left) ? cvt<Acc>(xt[c + e]) : Acc(0);
    }
  }
}
template <class O, class Acc, int VEC, int THREADS, int NV>
__device__ __forceinline__ void scan_tile_store_full(O* ot, const Acc (&v)[NV][VEC], const Acc (&add)[NV]) {
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    Vec<O, VEC> tv;
#pragma unroll
    for (int e = 0; e < VEC; ++e) tv.v[e] = cvt<O>((Acc)(v[k][e] + add[k]));
    vec_store<O, VEC, true>(ot + ((int64_t)k * THREADS + threadIdx.x) * VEC, tv);
  }
}
template <class O, class Acc, int VEC, int THREADS, int NV>
__device__ __forceinline__ void scan_tile_store(O* ot, int64_t left, const Acc (&v)[NV][VEC], const Acc (&add)[NV]) {
  if (left >= (int64_t)THREADS * NV * VEC) {
    scan_tile_store_full<O, Acc, VEC, THREADS, NV>(ot, v, add);
  } else {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int64_t c = ((int64_t)k * THREADS + threadIdx.x) * VEC;
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (c + e < left) ot[c + e] = cvt<O>((Acc)(v[k][e] + add[k]));
    }
  }
}

// THREADS is 256 or 1024.  Every workgroup draws one ticket from a single counter, and same-address atomics
// retire at roughly one per 12 ns on this chip, so a 16 KiB tile (256 lanes) caps the kernel near 2.7 TB/s of
// traffic; 64 KiB tiles (1024 lanes, same registers per lane) keep the ticket off the critical path.  The
// smaller tile is kept for inputs with too few tiles to fill the chip.
template <class T, class O, class Acc, int VEC, int THREADS, int NV>
__global__ __launch_bounds__(THREADS) void cumsum_lookback_kernel(const ScanArgs a) {
  constexpr int kTileElems = THREADS * NV * VEC;
  constexpr int kWaves = THREADS / kWave;
  constexpr int kTotals = NV * kWaves;          // wave totals of a tile, in tile order; one wave scans them
  static_assert(kTotals <= kWave, "wave 0 scans all wave totals in one pass");
  __shared__ Acc wave_tot[kTotals];              // first the totals, then their exclusive prefix sums
  __shared__ Acc tile_prefix;
  __shared__ unsigned int my_ticket;
  ScanHeader* hdr = (ScanHeader*)a.ws;
  unsigned long long* status = (unsigned long long*)(a.ws + 256);

  if (threadIdx.x == 0) my_ticket = atomicAdd(&hdr->ticket, 1u);
  __syncthreads();
  const int64_t ticket = my_ticket;
  if (ticket >= a.total_tiles) return;
  // tickets walk the rows round-robin (tile t of every row, then tile t + 1, ...): a tile's predecessors in its row
  // still have smaller tickets, and the workgroups resident at one time are spread over all rows instead of sitting
  // in one or two of them, which shortens every look-back chain
  const int64_t t = ticket / a.rows, row = ticket - t * a.rows;
  const int64_t slot = row * a.tiles_per_row + t;      // status word of this tile (row-major)
  const T* x = (const T*)a.x + row * a.xrow + t * kTileElems;
  O* out = (O*)a.out + row * a.orow + t * kTileElems;
  const int64_t left = a.len - t * kTileElems;      // valid elements in this tile (may exceed the tile)
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;

  Acc v[NV][VEC];
  scan_tile_load<T, Acc, VEC, THREADS, NV>(x, left, v);
  Acc excl[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
#pragma unroll
    for (int e = 1; e < VEC; ++e) v[k][e] += v[k][e - 1];
    const Acc incl = wave_inclusive(v[k][VEC - 1]);
    Acc up = shfl_up(incl, 1);
    excl[k] = lane == 0 ? Acc(0) : up;
    if (lane == kWave - 1) wave_tot[k * kWaves + w] = incl;     // tile order: sub-tile k, then wave w
  }
  __syncthreads();
  if (w == 0) {
    // exclusive scan of the wave totals, then the tile's exclusive prefix by look-back
    const Acc tot = lane < kTotals ? wave_tot[lane] : Acc(0);
    const Acc incl = wave_inclusive(tot);
    const Acc up = shfl_up(incl, 1);
    if (lane < kTotals) wave_tot[lane] = lane == 0 ? Acc(0) : up;
    const Acc tile_total = shfl_idx(incl, kTotals - 1);
    Acc prefix = Acc(0);
    if (t == 0) {
      if (lane == 0) TileState<Acc>::publish(status, slot, kPrefix, tile_total);
    } else {
      if (lane == 0) TileState<Acc>::publish(status, slot, kAggregate, tile_total);
      int64_t look = t - 1;                    // nearest predecessor not yet folded in (row-local index)
      bool done = false;
      while (!done) {
        const int64_t mine = look - lane;      // lane i inspects predecessor look - i
        Acc val = Acc(0);
        uint32_t flag = kPrefix;               // positions before the row start count as a zero prefix
        if (mine >= 0) {
          int spins = 0;
          do {
            flag = TileState<Acc>::read(status, slot - t + mine, &val);
            if (flag != kEmpty) break;
            __builtin_amdgcn_s_sleep(2);
          } while (++spins < kSpinLimit);
          if (flag == kEmpty) { hdr->error = 1; flag = kPrefix; val = Acc(0); }
        }
        const unsigned long long has_prefix = __ballot(flag == kPrefix);
        const int stop = __ffsll((long long)has_prefix) - 1;      // nearest predecessor holding a full prefix
        Acc contrib = (stop < 0 || lane <= stop) ? val : Acc(0);
#pragma unroll
        for (int m = kWave / 2; m >= 1; m >>= 1) contrib += shfl_xor(contrib, m);
        prefix += contrib;
        if (stop >= 0) done = true;
        else look -= kWave;
      }
      if (lane == 0) TileState<Acc>::publish(status, slot, kPrefix, prefix + tile_total);
    }
    if (lane == 0) tile_prefix = prefix;
  }
  __syncthreads();
  const Acc p = tile_prefix;
  Acc add[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) add[k] = p + wave_tot[k * kWaves + w] + excl[k];
  scan_tile_store<O, Acc, VEC, THREADS, NV>(out, left, v, add);
}

// Row-carry scan: one workgroup walks a whole row tile by tile and carries the running total in registers.
// No inter-workgroup traffic at all, so it is the better choice whenever there are enough rows to fill the
// chip.  The next tile's loads are issued before the current tile is scanned; for tiles that lie wholly
// inside the row every load and store is unconditional, so the wait for the prefetched tile can leave the
// previous tile's stores in flight.
template <class T, class O, class Acc, int VEC>
__global__ __launch_bounds__(kBlock) void cumsum_carry_kernel(const ScanArgs a) {
  constexpr int kTileElems = kBlock * kNV * VEC;
  constexpr int kWaves = kBlock / kWave;
  __shared__ Acc wave_tot[2][kNV][kWaves];
  const int64_t row = blockIdx.x;
  const T* x = (const T*)a.x + row * a.xrow;
  O* out = (O*)a.out + row * a.orow;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  Acc carry = Acc(0);
  Acc v[kNV][VEC], nxt[kNV][VEC];

  // scans the tile held in nxt (tile t).  steady == true: tiles t and t + 1 are both wholly inside the row, the
  // prefetch and the stores are branch-free; otherwise t + 1 may be ragged or absent.
  auto tile = [&](int64_t t, auto steady) {
#pragma unroll
    for (int k = 0; k < kNV; ++k)
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[k][e] = nxt[k][e];
    if constexpr (decltype(steady)::value)
      scan_tile_load_full<T, Acc, VEC, kBlock, kNV>(x + (t + 1) * kTileElems, nxt);
    else if (t + 1 < a.tiles_per_row)
      scan_tile_load<T, Acc, VEC, kBlock, kNV>(x + (t + 1) * kTileElems, a.len - (t + 1) * kTileElems, nxt);
    const int buf = (int)(t & 1);
    Acc excl[kNV];
#pragma unroll
    for (int k = 0; k < kNV; ++k) {
#pragma unroll
      for (int e = 1; e < VEC; ++e) v[k][e] += v[k][e - 1];
      const Acc incl = wave_inclusive(v[k][VEC - 1]);
      Acc up = shfl_up(incl, 1);
      excl[k] = lane == 0 ? Acc(0) : up;
      if (lane == kWave - 1) wave_tot[buf][k][w] = incl;
    }
    __syncthreads();                       // one barrier per tile: the two LDS buffers alternate
    Acc running = carry;
    Acc add[kNV];
#pragma unroll
    for (int k = 0; k < kNV; ++k) {
#pragma unroll
      for (int ww = 0; ww < kWaves; ++ww) {
        if (ww == w) add[k] = running + excl[k];
        running += wave_tot[buf][k][ww];
      }
    }
    carry = running;
    if constexpr (decltype(steady)::value) scan_tile_store_full<O, Acc, VEC, kBlock, kNV>(out + t * kTileElems, v, add);
    else scan_tile_store<O, Acc, VEC, kBlock, kNV>(out + t * kTileElems, a.len - t * kTileElems, v, add);
  };

  scan_tile_load<T, Acc, VEC, kBlock, kNV>(x, a.len, nxt);
  // The first tile must have landed before the steady loop is entered: otherwise the loop's own wait has to
  // cover "loads still pending, nothing issued after them" as well and becomes a full drain, which would also
  // sit out the previous tile's stores on every iteration.  (vmcnt = 0; the other counters are left alone.)
  __builtin_amdgcn_s_waitcnt(0x0F70);
  const int64_t nfull = a.len / kTileElems;          // tiles wholly inside the row: the branch-free path
  int64_t t = 0;
  for (; t + 1 < nfull; ++t) tile(t, std::true_type{});
  for (; t < a.tiles_per_row; ++t) tile(t, std::false_type{});
}

template <class T, class O, class Acc>
__global__ __launch_bounds__(kBlock) void cumsum_strided_kernel(const StridedArgs a) {
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (idx >= a.sl.count) return;
  int64_t xo, oo;
  slice_offsets(a.sl, idx, &xo, &oo);
  const T* x = (const T*)a.x + xo;
  O* out = (O*)a.out + oo;
  Acc acc = Acc(0);
  for (int64_t j = 0; j < a.len; ++j) {
    acc += cvt<Acc>(x[j * a.xs]);
    out[j * a.os] = cvt<O>(acc);
  }
}

struct ScanPlan {
  bool lookback;
  int vec;
  int64_t rows, len, xrow, orow, tiles_per_row, total_tiles;
  size_t ws_bytes;
};

template <class T, class O, class Acc> ScanPlan scan_plan(const tx_tensor* out, const tx_tensor* x, int dim, const Slices& sl) {
  constexpr int V = 16 / sizeof(T);
  ScanPlan p;
  memset(&p, 0, sizeof(p));
  const int nd = x->ndim;
  p.len = nd ? x->sizes[dim] : 1;
  const int64_t xs = nd ? x->strides[dim] : 1, os = nd ? out->strides[dim] : 1;
  p.lookback = p.len > 1 && xs == 1 && os == 1 && sl.n <= 1;
  if (!p.lookback) return p;
  p.rows = sl.count;
  p.xrow = sl.n ? sl.xs[0] : 0;
  p.orow = sl.n ? sl.os[0] : 0;
  constexpr int out_al = V * sizeof(O) >= 16 ? 16 : V * sizeof(O);
  const bool al = (uintptr_t)x->data % 16 == 0 && (uintptr_t)out->data % out_al == 0 &&
                  (p.xrow * (int64_t)sizeof(T)) % 16 == 0 && (p.orow * (int64_t)sizeof(O)) % out_al == 0;
  p.vec = al ? V : 1;
  const int64_t tile = (int64_t)kBlock * kNV * p.vec;
  p.tiles_per_row = (p.len + tile - 1) / tile;
  p.total_tiles = p.tiles_per_row * p.rows;
  p.ws_bytes = 256 + (size_t)p.total_tiles * TileState<Acc>::words * 8;
  return p;
}

template <class T, class O, class Acc>
tx_status cumsum_launch(const tx_tensor* out, const tx_tensor* x, int dim, void* ws, size_t ws_bytes, hipStream_t stream,
                        size_t* query) {
  constexpr int V = 16 / sizeof(T);
  Slices sl;
  build_slices(&sl, x, out, x->ndim ? dim : -1);
  ScanPlan p = scan_plan<T, O, Acc>(out, x, dim, sl);
  if (!p.lookback && x->ndim && strcmp(forced_path(), "scan-strided") && cols_path_ok(out, x, dim))
    return cumsum_cols(out, x, dim, ws, ws_bytes, stream, query);
  if (query) { *query = p.lookback ? p.ws_bytes : 0; return TX_OK; }
  if (sl.count >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "cumsum: too many slices");
  if (p.lookback) {
    if (p.total_tiles >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "cumsum: too many tiles");
    if (!ws || ws_bytes < p.ws_bytes)
      return fail(TX_ERR_WORKSPACE, "cumsum needs %zu workspace bytes, got %zu", p.ws_bytes, ws_bytes);
    if ((uintptr_t)ws % 8) return fail(TX_ERR_WORKSPACE, "cumsum workspace must be 8-byte aligned");
    ScanArgs a;
    a.x = (const char*)x->data;
    a.out = (char*)out->data;
    a.ws = (char*)ws;
    a.rows = p.rows;
    a.len = p.len;
    a.xrow = p.xrow;
    a.orow = p.orow;
    a.tiles_per_row = p.tiles_per_row;
    a.total_tiles = p.total_tiles;
    // short rows, and enough of them to fill the chip: one workgroup per row with a register carry.  Longer rows
    // go to the look-back scan, which spreads every row over many workgroups (on [4096,65536] it measured
    // 363 us against 397 us for the row-carry kernel, int64 756 against 809)
    bool carry = p.tiles_per_row == 1 || (p.rows >= 1024 && p.tiles_per_row <= 4);
    if (!strncmp(forced_path(), "scan-lookback", 13)) carry = false;
    if (!strcmp(forced_path(), "scan-carry")) carry = true;
    if (carry) {
      set_path(p.vec > 1 ? "scan-carry" : "scan-carry-scalar");
      if (p.vec > 1)
        hipLaunchKernelGGL((cumsum_carry_kernel<T, O, Acc, V>), dim3((unsigned)p.rows), dim3(kBlock), 0, stream, a);
      else
        hipLaunchKernelGGL((cumsum_carry_kernel<T, O, Acc, 1>), dim3((unsigned)p.rows), dim3(kBlock), 0, stream, a);
      return check_launch("cumsum row-carry kernel");
    }
    // 64 KiB tiles once the 16 KiB tiling has enough tiles for the ticket counter to be the limit
    constexpr int kBig = 1024, kBigNV = 4;
    const bool big = p.total_tiles >= 2048 && strcmp(forced_path(), "scan-lookback-narrow") != 0;
    if (big) {
      const int64_t tile = (int64_t)kBig * kBigNV * p.vec;
      a.tiles_per_row = (p.len + tile - 1) / tile;
      a.total_tiles = a.tiles_per_row * p.rows;
    }
    const int64_t words = (int64_t)((256 + (size_t)a.total_tiles * TileState<Acc>::words * 8) / 8);   // <= p.ws_bytes / 8
    hipLaunchKernelGGL(scan_clear_kernel, dim3((unsigned)((words + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream,
                       (unsigned long long*)ws, words);
    set_path(p.vec > 1 ? (big ? "scan-lookback-wide" : "scan-lookback") : (big ? "scan-lookback-wide-scalar" : "scan-lookback-scalar"));
    const dim3 grid((unsigned)a.total_tiles);
    if (p.vec > 1 && big)
      hipLaunchKernelGGL((cumsum_lookback_kernel<T, O, Acc, V, kBig, kBigNV>), grid, dim3(kBig), 0, stream, a);
    else if (p.vec > 1)
      hipLaunchKernelGGL((cumsum_lookback_kernel<T, O, Acc, V, kBlock, kNV>), grid, dim3(kBlock), 0, stream, a);
    else if (big)
      hipLaunchKernelGGL((cumsum_lookback_kernel<T, O, Acc, 1, kBig, kBigNV>), grid, dim3(kBig), 0, stream, a);
    else
      hipLaunchKernelGGL((cumsum_lookback_kernel<T, O, Acc, 1, kBlock, kNV>), grid, dim3(kBlock), 0, stream, a);
    return check_launch("cumsum look-back kernel");
  }
  StridedArgs a;
  a.x = (const char*)x->data;
  a.out = (char*)out->data;
  a.sl = sl;
  a.len = x->ndim ? x->sizes[dim] : 1;
  a.xs = x->ndim ? x->strides[dim] : 1;
  a.os = x->ndim ? out->strides[dim] : 1;
  a.is_log = 0;
  set_path("scan-strided");
  hipLaunchKernelGGL((cumsum_strided_kernel<T, O, Acc>), dim3((unsigned)((sl.count + kBlock - 1) / kBlock)), dim3(kBlock),
                     0, stream, a);
  return check_launch("cumsum strided kernel");
}

tx_status cumsum_dispatch(const tx_tensor* out, const tx_tensor* x, int dim, void* ws, size_t wsb, hipStream_t s,
                          size_t* query) {
  const bool wide = out->dtype == TX_F32;
  switch (x->dtype) {
    case TX_BOOL: return cumsum_launch<uint8_t, int64_t, int64_t>(out, x, dim, ws, wsb, s, query);
    case TX_I32: return cumsum_launch<int32_t, int64_t, int64_t>(out, x, dim, ws, wsb, s, query);
    case TX_I64: return cumsum_launch<int64_t, int64_t, int64_t>(out, x, dim, ws, wsb, s, query);
    case TX_F32: return cumsum_launch<float, float, float>(out, x, dim, ws, wsb, s, query);
    case TX_BF16:
      return wide ? cumsum_launch<bf16, float, float>(out, x, dim, ws, wsb, s, query)
                  : cumsum_launch<bf16, bf16, float>(out, x, dim, ws, wsb, s, query);
    default:
      return wide ? cumsum_launch<f16, float, float>(out, x, dim, ws, wsb, s, query)
                  : cumsum_launch<f16, f16, float>(out, x, dim, ws, wsb, s, query);
  }
}

tx_status rowop_checks(const char* name, const tx_tensor* out, const tx_tensor* x, int64_t dim, int* d, bool softmax) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x"))) return rc;
  const bool flt = dtype_is_float(x->dtype);
  if (softmax) {
    if (!flt) return fail(TX_ERR_DTYPE, "%s takes floating dtypes only", name);
    if (out->dtype != x->dtype && out->dtype != TX_F32) return fail(TX_ERR_DTYPE, "%s: out dtype", name);
  } else if (flt) {
    if (out->dtype != x->dtype && out->dtype != TX_F32) return fail(TX_ERR_DTYPE, "%s: out dtype", name);
  } else if (out->dtype != TX_I64) {
    return fail(TX_ERR_DTYPE, "%s of bool / integer input returns int64", name);
  }
  if (!same_sizes(out, x->ndim, x->sizes)) return fail(TX_ERR_SHAPE, "%s: out must have x's shape", name);
  if ((rc = wrap_dim(dim, x->ndim, d))) return rc;
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  if (partial_overlap(out, x) || (out->data == x->data && numel(x) > 0))
    return fail(TX_ERR_OVERLAP, "%s: out must not alias x", name);
  return TX_OK;
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

tx_status tx_softmax(const tx_tensor* out, const tx_tensor* x, int64_t dim, int is_log, void* stream) {
  int d;
  tx_status rc = rowop_checks("softmax", out, x, dim, &d, true);
  if (rc) return rc;
  set_path("");
  if (numel(x) == 0) return TX_OK;
  hipStream_t s = as_stream(stream);
  const bool wide = out->dtype == TX_F32;
  switch (x->dtype) {
    case TX_F32: return softmax_launch<float, float>(out, x, d, is_log, s);
    case TX_BF16: return wide ? softmax_launch<bf16, float>(out, x, d, is_log, s) : softmax_launch<bf16, bf16>(out, x, d, is_log, s);
    default: return wide ? softmax_launch<f16, float>(out, x, d, is_log, s) : softmax_launch<f16, f16>(out, x, d, is_log, s);
  }
}

tx_status tx_cumsum(const tx_tensor* out, const tx_tensor* x, int64_t dim, void* ws, size_t ws_bytes, void* stream) {
  int d;
  tx_status rc = rowop_checks("cumsum", out, x, dim, &d, false);
  if (rc) return rc;
  set_path("");
  if (numel(x) == 0) return TX_OK;
  return cumsum_dispatch(out, x, d, ws, ws_bytes, as_stream(stream), nullptr);
}

size_t tx_cumsum_workspace_bytes(const tx_tensor* out, const tx_tensor* x, int64_t dim) {
  int d;
  if (rowop_checks("cumsum", out, x, dim, &d, false)) return 0;
  if (numel(x) == 0) return 0;
  size_t q = 0;
  cumsum_dispatch(out, x, d, nullptr, 0, nullptr, &q);
  return q;
}

}  // extern "C"
