// Indexing operators: gather, index_select, scatter_add_.
//
//   index_select : when the slice below `dim` is one contiguous, 16-byte
//                  granular run in both src and out, a wave copies whole
//                  slices with 16-byte lanes (several slices in flight per
//                  wave); otherwise one lane per output element.
//   gather       : one lane per output element (index reads are coalesced,
//                  the src reads are data-dependent).
//   scatter_add_ : integer / bool dtypes use device atomics (order-free, so
//                  exact).  Floating dtypes, deterministic: the (destination,
//                  position) pairs are radix-sorted by destination (stable,
//                  so positions stay ascending), then summed per destination
//                  in a fixed order.  When the index is a row id broadcast
//                  over the trailing dims ("row mode": whole rows of src go
//                  to rows of self) the sort runs over rows only and a wave
//                  sums a chunk of sorted rows with 16-byte lanes; long runs
//                  are cut at fixed chunk boundaries and their partial rows
//                  combined in chunk order, so the association order depends
//                  on the data alone.
#include <algorithm>
#include <cstring>
#include <limits>

#include "common.h"
#include "index_util.h"

namespace tx {
namespace {

constexpr int kBlock = 256;



// ---------------------------------------------------------------------------
// gather / generic index_select / atomic scatter_add share one addressing
// scheme: iterate a shape (the index's, or out's), compute up to three
// strided offsets, and replace coordinate `dim` for one operand by the index.
// ---------------------------------------------------------------------------
struct ElemArgs {
  Dims shape;
  int dim;
  int index_is64;
  const char* index;
  const char* src;
  char* dst;
  int64_t istride[TX_MAX_DIMS];    // index strides (index_select: only [dim] is used)
  int64_t sstride[TX_MAX_DIMS];    // source strides
  int64_t dstride[TX_MAX_DIMS];    // destination strides
  float alpha_f;                   // scatter / index_add: multiplier of the source (floating dtypes)
  int64_t alpha_i;                 // the same for integer dtypes (wrapping); bool: zero or not
  int64_t wrap;                    // scatter: added to a negative index (0: indices are never negative)
};

// alpha * v in the arithmetic of T (sums are linear, so the sorted paths scale a whole sum once)
template <class T, class V> __device__ __forceinline__ V scaled(V v, float alpha_f, int64_t alpha_i) {
  if constexpr (std::is_same<T, uint8_t>::value) return alpha_i ? v : V(0);
  else if constexpr (std::is_integral<T>::value) return (V)((unsigned long long)v * (unsigned long long)alpha_i);
  else return v * (V)alpha_f;
}

// Each lane handles kGatherU elements (a workgroup covers kGatherU consecutive runs of 256): all index loads
// are issued first, then all data-dependent source loads, so several random accesses are in flight per lane.
// (Every random 4-byte element costs a 128-byte read from HBM; loading it with system scope - the sc0 sc1 bits, an
// L2 bypass - changes neither the request size, still 4.44 M requests of 128 bytes for 4.19 M elements, nor the time.)
constexpr int kGatherU = 4;
template <class B>
__global__ __launch_bounds__(kBlock) void gather_kernel(const ElemArgs a, int index_1d) {
  int64_t so[kGatherU], d_o[kGatherU], k[kGatherU];
  bool live[kGatherU];
#pragma unroll
  for (int u = 0; u < kGatherU; ++u) {
    const int64_t lin = ((int64_t)blockIdx.x * kGatherU + u) * kBlock + threadIdx.x;
    live[u] = lin < a.shape.numel;
    int64_t io = 0, dimcoord = 0;
    so[u] = 0;
    d_o[u] = 0;
    k[u] = 0;
    if (!live[u]) continue;
    uint32_t rem = (uint32_t)lin;
    for (int d = a.shape.n - 1; d >= 0; --d) {
      uint32_t q, m;
      a.shape.div[d].divmod(rem, q, m);
      rem = q;
      d_o[u] += (int64_t)m * a.dstride[d];
      if (d == a.dim) dimcoord = m;
      else so[u] += (int64_t)m * a.sstride[d];
      if (!index_1d) io += (int64_t)m * a.istride[d];
    }
    if (index_1d) io = dimcoord * a.istride[a.dim];
    k[u] = load_index(a.index, io, a.index_is64);
  }
  B v[kGatherU];
#pragma unroll
  for (int u = 0; u < kGatherU; ++u)
    if (live[u]) v[u] = ((const B*)a.src)[so[u] + k[u] * a.sstride[a.dim]];
#pragma unroll
  for (int u = 0; u < kGatherU; ++u)
    if (live[u]) ((B*)a.dst)[d_o[u]] = v[u];
}

// index_select fast path: slice r = (outer o, picked j) is `vecs` 16-byte vectors
struct RowCopyArgs {
  const char* index;
  const char* src;
  char* dst;
  int index_is64;
  int64_t istride;
  int64_t nsel;               // number of indices
  FastDiv nsel_div;
  int64_t rows;               // outer * nsel
  int64_t src_outer, dst_outer;   // byte strides of the outer dim
  int64_t src_dim, dst_dim;       // byte strides of `dim`
  int64_t vecs;               // 16-byte vectors per slice
};

constexpr int kRowsPerWave = 2;

// One wave copies 2 selected slices at a time, 16 bytes per lane (measured on 4 Mi rows of 1 KiB: 1294 us with 2
// slices per wave, 1342 with 4, 1452 with 8 - many small waves stream best on this chip).  Lane i resolves slice r0 + i (index
// load, offsets) and the byte offsets are handed out with readlane, so the copy loop has no index
// dependence; slices past the end are clamped to the last one (the same bytes are then written twice),
// which keeps every load and store unconditional and their number known at compile time.
__global__ __launch_bounds__(kBlock) void index_select_rows_kernel(const RowCopyArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * (kBlock / kWave) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int64_t r0 = wave * kRowsPerWave;
  if (r0 >= a.rows) return;
  int64_t so, d_o;
  {
    const int64_t r = std::min<int64_t>(r0 + (lane < kRowsPerWave ? lane : 0), a.rows - 1);
    uint32_t o, j;
    a.nsel_div.divmod((uint32_t)r, o, j);
    const int64_t k = load_index(a.index, (int64_t)j * a.istride, a.index_is64);
    so = (int64_t)o * a.src_outer + k * a.src_dim;
    d_o = (int64_t)o * a.dst_outer + (int64_t)j * a.dst_dim;
  }
  auto lane_value = [&](int64_t v, int i) -> int64_t {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, i);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), i);
    return (int64_t)(((uint64_t)hi << 32) | lo);
  };
  const u32x4* sp[kRowsPerWave];
  u32x4* dp[kRowsPerWave];
#pragma unroll
  for (int i = 0; i < kRowsPerWave; ++i) {
    sp[i] = (const u32x4*)(a.src + lane_value(so, i));
    dp[i] = (u32x4*)(a.dst + lane_value(d_o, i));
  }
  for (int64_t v = lane; v < a.vecs; v += kWave) {
    u32x4 t[kRowsPerWave];
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) t[i] = sp[i][v];                          // selected rows may be read again (non-temporal: 1490 against 1355 us)
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) __builtin_nontemporal_store(t[i], dp[i] + v);   // the output is written once
  }
}

// ---------------------------------------------------------------------------
// scatter_add with atomics
// ---------------------------------------------------------------------------
template <class T> __device__ __forceinline__ void atomic_accumulate(T* p, T v);
template <> __device__ __forceinline__ void atomic_accumulate<int32_t>(int32_t* p, int32_t v) { atomicAdd(p, v); }
template <> __device__ __forceinline__ void atomic_accumulate<int64_t>(int64_t* p, int64_t v) {
  atomicAdd((unsigned long long*)p, (unsigned long long)v);
}
template <> __device__ __forceinline__ void atomic_accumulate<float>(float* p, float v) { atomicAdd(p, v); }
template <> __device__ __forceinline__ void atomic_accumulate<uint8_t>(uint8_t* p, uint8_t v) {
  if (!v) return;
  const uintptr_t addr = (uintptr_t)p;
  unsigned int* word = (unsigned int*)(addr & ~(uintptr_t)3);
  atomicOr(word, 1u << (8 * (addr & 3)));
}
template <class T>
__global__ __launch_bounds__(kBlock) void scatter_add_atomic_kernel(const ElemArgs a) {
  const int64_t lin = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (lin >= a.shape.numel) return;
  int64_t io = 0, so = 0, d_o = 0;
  uint32_t rem = (uint32_t)lin;
  for (int d = a.shape.n - 1; d >= 0; --d) {
    uint32_t q, m;
    a.shape.div[d].divmod(rem, q, m);
    rem = q;
    io += (int64_t)m * a.istride[d];
    so += (int64_t)m * a.sstride[d];
    if (d != a.dim) d_o += (int64_t)m * a.dstride[d];
  }
  int64_t k = load_index(a.index, io, a.index_is64);
  k += k < 0 ? a.wrap : 0;
  d_o += k * a.dstride[a.dim];
  atomic_accumulate<T>((T*)a.dst + d_o, scaled<T, T>(((const T*)a.src)[so], a.alpha_f, a.alpha_i));
}

// ---------------------------------------------------------------------------
// stable LSD radix sort of (key, value) pairs, 8 bits per pass
// ---------------------------------------------------------------------------
constexpr int kSortItems = 8;
constexpr int kSortTile = kBlock * kSortItems;          // 2048 entries per workgroup
constexpr int kWaves = kBlock / kWave;

// keys for the element mode: destination element offset of every index position.  The value that travels with a key
// is the position (EB = 0) or, for sources of EB = 1, 2 or 4 bytes, the source element itself, zero-extended: the
// sort is stable, so values of equal keys stay in position order and the reduction needs no gather afterwards.
template <int EB>
__global__ __launch_bounds__(kBlock) void scatter_keys_kernel(const ElemArgs a, uint32_t* keys, uint32_t* vals) {
  const int64_t lin = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (lin >= a.shape.numel) return;
  int64_t io = 0, d_o = 0, so = 0;
  uint32_t rem = (uint32_t)lin;
  for (int d = a.shape.n - 1; d >= 0; --d) {
    uint32_t q, m;
    a.shape.div[d].divmod(rem, q, m);
    rem = q;
    io += (int64_t)m * a.istride[d];
    if (d != a.dim) d_o += (int64_t)m * a.dstride[d];
    if constexpr (EB != 0) so += (int64_t)m * a.sstride[d];
  }
  int64_t k = load_index(a.index, io, a.index_is64);
  k += k < 0 ? a.wrap : 0;
  d_o += k * a.dstride[a.dim];
  keys[lin] = (uint32_t)d_o;
  if constexpr (EB == 4) vals[lin] = ((const uint32_t*)a.src)[so];
  else if constexpr (EB == 2) vals[lin] = ((const uint16_t*)a.src)[so];
  else if constexpr (EB == 1) vals[lin] = ((const uint8_t*)a.src)[so];
  else vals[lin] = (uint32_t)lin;
}
template <class T> constexpr int key_value_bytes() { return sizeof(T) <= 4 ? (int)sizeof(T) : 0; }
template <class T> __device__ __forceinline__ T value_from_bits(uint32_t b) {
  if constexpr (sizeof(T) == 4) return __builtin_bit_cast(T, b);
  else if constexpr (sizeof(T) == 2) return __builtin_bit_cast(T, (uint16_t)b);
  else return __builtin_bit_cast(T, (uint8_t)b);
}
// The first pass of the row mode in one kernel: the row id of every source row becomes its key (and its position the
// value), and the tile's histogram of the lowest digit is counted from the keys while they are in registers.
__global__ __launch_bounds__(kBlock) void row_keys_hist_kernel(const char* index, int is64, int64_t istride, int64_t n,
                                                               uint32_t* keys, uint32_t* vals, unsigned int* counter,
                                                               int64_t wrap, uint32_t* hist, int nblocks) {
  __shared__ unsigned int h[256];
  h[threadIdx.x] = 0;
  if (blockIdx.x == 0 && threadIdx.x < 2 && counter) counter[threadIdx.x] = 0u;      // lengths of the start list and the long-run list of the row-mode combine pass
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
  for (int k = 0; k < kSortItems; ++k) {
    const int64_t i = base + k * kBlock + threadIdx.x;
    if (i < n) {
      int64_t key = load_index(index, i * istride, is64);
      key += key < 0 ? wrap : 0;
      keys[i] = (uint32_t)key;
      vals[i] = (uint32_t)i;
      atomicAdd(&h[(uint32_t)key & 255u], 1u);
    }
  }
  __syncthreads();
  hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(kBlock) void sort_hist_kernel(const uint32_t* keys, int64_t n, int shift, uint32_t* hist,
                                                           int nblocks) {
  __shared__ unsigned int h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
  for (int k = 0; k < kSortItems; ++k) {
    const int64_t i = base + k * kBlock + threadIdx.x;
    if (i < n) atomicAdd(&h[(keys[i] >> shift) & 255u], 1u);
  }
  __syncthreads();
  hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

// one workgroup per digit: exclusive scan of that digit's per-block counts, plus the digit total
__global__ __launch_bounds__(kBlock) void sort_rowscan_kernel(uint32_t* hist, int nblocks, uint32_t* totals) {
  __shared__ unsigned int wsum[kWaves];
  __shared__ unsigned int carry;
  uint32_t* row = hist + (int64_t)blockIdx.x * nblocks;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < nblocks; base += kBlock) {
    const int i = base + threadIdx.x;
    const unsigned int v = i < nblocks ? row[i] : 0u;
    unsigned int incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      unsigned int o = __shfl_up(incl, d, kWave);
      if (lane >= d) incl += o;
    }
    if (lane == kWave - 1) wsum[w] = incl;
    __syncthreads();
    unsigned int before = carry;
    for (int ww = 0; ww < w; ++ww) before += wsum[ww];
    if (i < nblocks) row[i] = before + incl - v;
    __syncthreads();
    if (threadIdx.x == kBlock - 1) carry = before + incl;
    __syncthreads();
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

__global__ __launch_bounds__(kBlock) void sort_scatter_kernel(const uint32_t* keys_in, const uint32_t* vals_in,
                                                              uint32_t* keys_out, uint32_t* vals_out, int64_t n, int shift,
                                                              const uint32_t* hist, const uint32_t* totals, int nblocks) {
  __shared__ unsigned int digit_base[256];
  __shared__ unsigned int cnt[kWaves][256];
  __shared__ unsigned int wsum[kWaves];
  __shared__ unsigned int tile_start[256];
  __shared__ uint32_t tile_key[kSortTile], tile_val[kSortTile];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  {  // exclusive scan of the 256 digit totals
    const unsigned int v = totals[threadIdx.x];
    unsigned int incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      unsigned int o = __shfl_up(incl, d, kWave);
      if (lane >= d) incl += o;
    }
    if (lane == kWave - 1) wsum[w] = incl;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) cnt[ww][threadIdx.x] = 0;
    __syncthreads();
    unsigned int before = 0;
    for (int ww = 0; ww < w; ++ww) before += wsum[ww];
    digit_base[threadIdx.x] = before + incl - v;
  }
  __syncthreads();
  // wave w owns entries [base + w*512, +512) as 8 runs of 64, taken in order
  const int64_t base = (int64_t)blockIdx.x * kSortTile + (int64_t)w * (kWave * kSortItems);
  uint32_t key[kSortItems], val[kSortItems], off[kSortItems];
  const unsigned long long lt = (1ull << lane) - 1ull;
#pragma unroll
  for (int s = 0; s < kSortItems; ++s) {
    const int64_t i = base + s * kWave + lane;
    const bool valid = i < n;
    key[s] = valid ? keys_in[i] : 0u;
    val[s] = valid ? vals_in[i] : 0u;
    const uint32_t dg = (key[s] >> shift) & 255u;
    unsigned long long peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const unsigned long long bal = __ballot((dg >> b) & 1u);
      peers &= ((dg >> b) & 1u) ? bal : ~bal;
    }
    const unsigned int rank = __popcll(peers & lt);
    unsigned int old = 0;
    if (valid) old = cnt[w][dg];
    __builtin_amdgcn_wave_barrier();
    if (valid && rank == 0) cnt[w][dg] = old + __popcll(peers);
    __builtin_amdgcn_wave_barrier();
    off[s] = old + rank;
  }
  __syncthreads();
  // Order the tile in LDS first, so that neighbouring lanes then store to neighbouring addresses of a digit's range.
  {  // one lane per digit: where the digit starts in the ordered tile, and what to add to get its place in the output
    unsigned int v = 0;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) v += cnt[ww][threadIdx.x];
    unsigned int incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      unsigned int o = __shfl_up(incl, d, kWave);
      if (lane >= d) incl += o;
    }
    if (lane == kWave - 1) wsum[w] = incl;
    __syncthreads();
    unsigned int before = 0;
    for (int ww = 0; ww < w; ++ww) before += wsum[ww];
    const unsigned int start = before + incl - v;
    tile_start[threadIdx.x] = start;
    digit_base[threadIdx.x] += hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] - start;
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < kSortItems; ++s) {
    const int64_t i = base + s * kWave + lane;
    if (i < n) {
      const uint32_t dg = (key[s] >> shift) & 255u;
      unsigned int pos = tile_start[dg] + off[s];
      for (int ww = 0; ww < w; ++ww) pos += cnt[ww][dg];
      tile_key[pos] = key[s];
      tile_val[pos] = val[s];
    }
  }
  __syncthreads();
  const int64_t tile_base = (int64_t)blockIdx.x * kSortTile;
  const int nvalid = (int)std::min<int64_t>(kSortTile, n - tile_base);
#pragma unroll
  for (int s = 0; s < kSortItems; ++s) {
    const int i = s * kBlock + threadIdx.x;
    if (i < nvalid) {
      const uint32_t kk = tile_key[i];
      const unsigned int pos = digit_base[(kk >> shift) & 255u] + i;
      keys_out[pos] = kk;
      vals_out[pos] = tile_val[i];
    }
  }
}

// ---------------------------------------------------------------------------
// deterministic segmented reductions
// ---------------------------------------------------------------------------
// Element mode (scatter_reduce_ in every mode; the float sums of scatter_add_ / index_put_ with an index that is not
// a broadcast row id): runs of equal keys are combined in position order (binary64 for floats, wrapping 64-bit for
// integers), then with the element's own value when it is included.
enum { kRedSum = 0, kRedProd = 1, kRedMean = 2, kRedAmax = 3, kRedAmin = 4 };
enum { kNone = 0, kEnd = 1, kThrough = 2 };       // what the piece at the start of a chunk or block does

// scatter_reduce_ on the element-key sort.  The sorted (destination element, position) pairs are cut into blocks of
// kBlock entries, one per workgroup; a run of equal keys is cut where it crosses a block boundary, and each piece is
// combined in binary64 / wrapping int64.  A run that lies inside one block is finished there.  The pieces of a run that crosses blocks are parked - the piece that ends a block in part_b, the
// piece that begins a block in part_a with a mark saying whether the run stops in that block or passes through it -
// and seg_reduce_finish_kernel adds them up in block order, one lane per crossing run.  Inside a block the pieces
// come from a segmented scan (every lane gathers its own value; shuffles inside a wave, then the waves' last pieces), so the association of
// a floating-point sum is a tree within a block and left to right across blocks; it depends only on the data.
template <class A> struct RedPart {
  A acc;
  int64_t count;
};
template <class T> struct RedOps {
  using A = typename std::conditional<std::is_integral<T>::value, int64_t, double>::type;
  __device__ __forceinline__ static A combine(int mode, A x, A v) {
    if constexpr (std::is_integral<T>::value) {
      switch (mode) {
        case kRedProd: return (A)((uint64_t)x * (uint64_t)v);
        case kRedAmax: return v > x ? v : x;
        case kRedAmin: return v < x ? v : x;
        default: return (A)((uint64_t)x + (uint64_t)v);
      }
    } else {
      switch (mode) {
        case kRedProd: return x * v;
        case kRedAmax: return (x != x || v != v) ? (A)__builtin_nan("") : (v > x ? v : x);
        case kRedAmin: return (x != x || v != v) ? (A)__builtin_nan("") : (v < x ? v : x);
        default: return x + v;
      }
    }
  }
  // folds in the destination's own value if asked, divides for the mean, stores
  __device__ __forceinline__ static void finish(int mode, int include_self, T* dst, A acc, int64_t count, float alpha = 1.0f) {
    if constexpr (!std::is_integral<T>::value)
      if (mode == kRedSum) acc *= (double)alpha;        // scatter_add_ / index_add_ scale the sum of what arrives
    if (include_self) {
      acc = combine(mode, acc, cvt<A>(*dst));
      ++count;
    }
    if constexpr (std::is_integral<T>::value) {
      if constexpr (std::is_same<T, uint8_t>::value) acc = acc != 0;     // bool: a sum of ones is an OR
      else acc = (A)(T)acc;                              // int32 arithmetic wraps at 32 bits (before a mean divides)
      if (mode == kRedMean) {                            // rounding toward -infinity
        A q = acc / count;
        if (acc % count != 0 && acc < 0) --q;
        acc = q;
      }
      *dst = (T)acc;
    } else {
      if (mode == kRedMean) acc /= (double)count;
      *dst = cvt<T>((float)acc);                         // binary64 -> fp32 -> T: T is fp32 or narrower
    }
  }
};
struct RedPieces {                                       // per block of kBlock sorted entries
  char* part_a;                                          // RedPart: the piece that begins the block and continues a run
  char* part_b;                                          // RedPart: the piece that ends the block and goes on
  uint8_t* flag_a;                                       // kNone / kEnd / kThrough for part_a
};

template <class T, bool BITS>                            // BITS: vals holds the source elements, not their positions
__global__ __launch_bounds__(kBlock) void seg_reduce_kernel(const uint32_t* keys, const uint32_t* vals, int64_t n,
                                                            const ElemArgs a, int mode, int include_self, RedPieces pc) {
  using A = typename RedOps<T>::A;
  __shared__ A sh_acc[kBlock / 64];
  __shared__ int sh_cnt[kBlock / 64];
  __shared__ uint32_t sh_key[kBlock / 64];
  const int t = threadIdx.x;
  const int64_t j = (int64_t)blockIdx.x * kBlock + t;
  const bool valid = j < n;
  const int64_t jc = valid ? j : n - 1;                  // lanes past the end read the last entry and store nothing
  const uint32_t k = keys[jc];
  A acc;
  if constexpr (BITS && sizeof(T) <= 4) {
    acc = cvt<A>(value_from_bits<T>(vals[jc]));
  } else {
    int64_t so = 0;
    uint32_t rem = vals[jc];
    for (int d = a.shape.n - 1; d >= 0; --d) {
      uint32_t q, m;
      a.shape.div[d].divmod(rem, q, m);
      rem = q;
      so += (int64_t)m * a.sstride[d];
    }
    acc = cvt<A>(((const T*)a.src)[so]);
  }
  int cnt = 1;
  // Segmented inclusive scan over the block's entries.  Keys are sorted, so the entry d places back belongs to the
  // same run exactly when its key is equal; the earlier operand always goes on the left.
  const int lane = t & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t ko = shfl_up(k, d);
    const A ao = shfl_up(acc, d);
    const int co = shfl_up(cnt, d);
    if (lane >= d && ko == k) {
      acc = RedOps<T>::combine(mode, ao, acc);
      cnt += co;
    }
  }
  // across waves: the last lane of a wave holds the piece that ends it; a lane whose run reaches back to the start of
  // its wave takes in the pieces of the waves before, nearest first, for as long as they carry the same key whole
  const int w = t >> 6;
  if (lane == 63) {
    sh_acc[w] = acc;
    sh_cnt[w] = cnt;
    sh_key[w] = k;
  }
  __syncthreads();
  if (cnt == lane + 1) {
    A carry = A(0);
    int ccnt = 0;
    for (int p = w - 1; p >= 0 && sh_key[p] == k; --p) {
      carry = ccnt ? RedOps<T>::combine(mode, sh_acc[p], carry) : sh_acc[p];
      ccnt += sh_cnt[p];
      if (sh_cnt[p] != 64) break;
    }
    if (ccnt) {
      acc = RedOps<T>::combine(mode, carry, acc);
      cnt += ccnt;
    }
  }
  if (!valid) return;
  const bool ends_run = j + 1 == n || keys[j + 1] != k;
  if (t == 0 && (j == 0 || keys[j - 1] != k)) pc.flag_a[blockIdx.x] = kNone;
  if (!ends_run && t != kBlock - 1) return;              // a piece ends where a run ends, and at the block's last entry
  const int first = t - cnt + 1;                         // where this piece begins in the block
  const bool starts_run = first > 0 || j - t == 0 || keys[j - t - 1] != k;
  if (starts_run && ends_run) {
    RedOps<T>::finish(mode, include_self, (T*)a.dst + k, acc, (int64_t)cnt, a.alpha_f);
  } else if (!starts_run) {
    ((RedPart<A>*)pc.part_a)[blockIdx.x] = RedPart<A>{acc, (int64_t)cnt};
    pc.flag_a[blockIdx.x] = ends_run ? kEnd : kThrough;
  } else {
    ((RedPart<A>*)pc.part_b)[blockIdx.x] = RedPart<A>{acc, (int64_t)cnt};
  }
}

// one lane per block whose last piece starts a run that crosses into the next block
template <class T>
__global__ __launch_bounds__(kBlock) void seg_reduce_finish_kernel(const uint32_t* keys, int64_t n, int64_t nblocks, const ElemArgs a,
                                                                   int mode, int include_self, RedPieces pc) {
  using A = typename RedOps<T>::A;
  const int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (b >= nblocks) return;
  const int64_t last = std::min<int64_t>((b + 1) * kBlock, n) - 1;
  if (last + 1 >= n || keys[last + 1] != keys[last]) return;           // nothing crosses
  if (pc.flag_a[b] == kThrough) return;                                // the crossing run started before this block
  RedPart<A> r = ((const RedPart<A>*)pc.part_b)[b];
  for (int64_t bb = b + 1; bb < nblocks; ++bb) {
    const RedPart<A> piece = ((const RedPart<A>*)pc.part_a)[bb];
    r.acc = RedOps<T>::combine(mode, r.acc, piece.acc);
    r.count += piece.count;
    if (pc.flag_a[bb] != kThrough) break;
  }
  RedOps<T>::finish(mode, include_self, (T*)a.dst + keys[last], r.acc, r.count, a.alpha_f);
}

// index_put_: one lane per element of the value shape I + rest.  MODE 0 assigns, 1 accumulates with an atomic
// (integers, bool), 2 only records the destination element offset as a sort key.
struct PutArgs {
  Dims shape;                        // I (the broadcast index shape) followed by the dims of self that are not indexed
  int nidx, ind;                     // index tensors; rank of I
  const char* index[TX_MAX_DIMS];
  int is64[TX_MAX_DIMS];
  int64_t istride[TX_MAX_DIMS][TX_MAX_DIMS];   // [index tensor][dim of I], 0 where it broadcasts
  int64_t extent[TX_MAX_DIMS];       // self.size(j) of the indexed dims (negative indices wrap)
  int64_t dstride_idx[TX_MAX_DIMS];  // self.stride(j) of the indexed dims
  int64_t dstride[TX_MAX_DIMS];      // per dim of `shape`: self's stride for the rest dims, 0 for the dims of I
  int64_t vstride[TX_MAX_DIMS];      // values' strides over `shape` (0 where it broadcasts)
  const char* src;
  char* dst;
  uint32_t* keys;
  uint32_t* vals;
};

template <class T, int MODE>
__global__ __launch_bounds__(kBlock) void index_put_kernel(const PutArgs a) {
  const int64_t lin = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (lin >= a.shape.numel) return;
  int64_t coord[TX_MAX_DIMS];
  int64_t vo = 0, d_o = 0;
  uint32_t rem = (uint32_t)lin;
  for (int d = a.shape.n - 1; d >= 0; --d) {
    uint32_t q, m;
    a.shape.div[d].divmod(rem, q, m);
    rem = q;
    coord[d] = m;
    vo += (int64_t)m * a.vstride[d];
    d_o += (int64_t)m * a.dstride[d];
  }
  for (int j = 0; j < a.nidx; ++j) {
    int64_t io = 0;
    for (int d = 0; d < a.ind; ++d) io += coord[d] * a.istride[j][d];
    int64_t k = load_index(a.index[j], io, a.is64[j]);
    k += k < 0 ? a.extent[j] : 0;
    d_o += k * a.dstride_idx[j];
  }
  if constexpr (MODE == 2) {
    a.keys[lin] = (uint32_t)d_o;
    a.vals[lin] = (uint32_t)lin;
  } else if constexpr (MODE == 1) {
    atomic_accumulate<T>((T*)a.dst + d_o, ((const T*)a.src)[vo]);
  } else {
    ((T*)a.dst)[d_o] = ((const T*)a.src)[vo];
  }
}

// index_put_ without accumulation, one 1-D index over dim 0 and whole contiguous rows: index_select_rows_kernel the
// other way round - source rows in order, destination rows picked by the index (negative indices wrap).  A row is
// `vecs` 16-byte vectors.  With duplicate indices the destination row receives one of the candidate rows' vectors,
// vector by vector, as it receives one of the candidates element by element on the general path.
struct RowPutArgs {
  const char* index;
  const char* src;
  char* dst;
  int index_is64;
  int64_t istride;
  int64_t rows;               // number of indices = source rows
  int64_t extent;             // self.size(0)
  int64_t src_row, dst_row;   // byte strides of dim 0
  int64_t vecs;
};
__global__ __launch_bounds__(kBlock) void index_put_rows_kernel(const RowPutArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * (kBlock / kWave) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int64_t r0 = wave * kRowsPerWave;
  if (r0 >= a.rows) return;
  int64_t so, d_o;
  {
    const int64_t r = std::min<int64_t>(r0 + (lane < kRowsPerWave ? lane : 0), a.rows - 1);    // clamped: the last row twice
    int64_t k = load_index(a.index, r * a.istride, a.index_is64);
    k += k < 0 ? a.extent : 0;
    so = r * a.src_row;
    d_o = k * a.dst_row;
  }
  auto lane_value = [&](int64_t v, int i) -> int64_t {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, i);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), i);
    return (int64_t)(((uint64_t)hi << 32) | lo);
  };
  const u32x4* sp[kRowsPerWave];
  u32x4* dp[kRowsPerWave];
#pragma unroll
  for (int i = 0; i < kRowsPerWave; ++i) {
    sp[i] = (const u32x4*)(a.src + lane_value(so, i));
    dp[i] = (u32x4*)(a.dst + lane_value(d_o, i));
  }
  for (int64_t v = lane; v < a.vecs; v += kWave) {
    u32x4 t[kRowsPerWave];
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) t[i] = __builtin_nontemporal_load(sp[i] + v);   // the values are read once
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) dp[i][v] = t[i];
  }
}

constexpr int kMaxChunk = 256;              // sorted rows per wave, at most
constexpr int64_t kIntRowModeMin = 4096;    // integer row mode pays for its sort from about this many rows
constexpr int kShortRun = 8;                // continuation pieces that one wave of the combine pass adds by itself
constexpr int kCombineBlocks = 2048;
constexpr int kLongWaves = 16;              // waves that share a run with more pieces
constexpr int kLongBlocks = 64;

// Sorted rows per wave.  Large inputs take 256 (half the boundary pieces of 128, and a bare row-summing loop measured
// 3 % faster); smaller ones take shorter chunks, so that the grid still covers the chip and a wave's chain of load
// round trips (one per 8 rows) stays short.  A function of n alone: the order of additions depends only on the data.
inline int seg_chunk(int64_t n) { return n >= 256 * 4096 ? 256 : n >= 128 * 4096 ? 128 : 64; }

struct SegRowArgs {
  const uint32_t* keys;
  const uint32_t* vals;
  int64_t n, nchunks;
  int chunk;                     // sorted rows per wave (seg_chunk)
  const char* src;
  char* self;
  int64_t src_row, self_row;     // element strides between rows
  int64_t width;                 // elements per row
  char* part_a;                  // [nchunks][width] accumulators: piece that continues from the previous chunk
  char* part_b;                  // [nchunks][width] accumulators: piece that continues into the next chunk
  uint8_t* flag_a;               // kNone / kEnd / kThrough
  uint32_t* key_b;               // destination row of the chunk's start piece
  uint32_t* start_list;          // chunks that hold the start piece of a run that goes on
  unsigned int* nstart;          // length of start_list (cleared by row_keys_hist_kernel)
  uint32_t* long_list;           // those of them whose run has more than kShortRun continuation pieces
  unsigned int* nlong;           // length of long_list (cleared by row_keys_hist_kernel)
  float alpha_f;                 // multiplier of every sum (floating dtypes / integer dtypes)
  int64_t alpha_i;
  int include_self;              // OP >= 0 kernels only: whether self takes part
};

// Accumulator of a segmented row sum: fp32 for the floating dtypes, wrapping unsigned arithmetic for integers.
template <class T> struct SegAcc { using type = float; };
template <> struct SegAcc<int32_t> { using type = uint32_t; };
template <> struct SegAcc<int64_t> { using type = unsigned long long; };
template <class T, class Acc> __device__ __forceinline__ T seg_add(T old, Acc sum) {
  if constexpr (std::is_integral<T>::value) return (T)((Acc)old + sum);
  else return cvt<T>(cvt<float>(old) + sum);
}

// OP >= 0 variants of the row kernels (scatter_reduce_ with a broadcast row index; OP = -1 is scatter_add_ with its
// multiplier): the same walk with the combining operator one of sum, amax and amin (all exact or order-insensitive enough for an fp32
// accumulator; prod and mean are not), and self taking part or not.  Integer accumulators hold the value's bits.
template <class T, class Acc, int OP> __device__ __forceinline__ Acc seg_identity() {
  if constexpr (OP != kRedAmax && OP != kRedAmin) return Acc(0);
  else if constexpr (std::is_integral<T>::value)
    return (Acc)(OP == kRedAmax ? std::numeric_limits<T>::lowest() : std::numeric_limits<T>::max());
  else return OP == kRedAmax ? -__builtin_inff() : __builtin_inff();
}
template <class T, class Acc, int OP> __device__ __forceinline__ Acc seg_op(Acc a, Acc v) {
  if constexpr (OP != kRedAmax && OP != kRedAmin) {
    return a + v;
  } else if constexpr (std::is_integral<T>::value) {
    const T x = (T)a, y = (T)v;
    return (Acc)(OP == kRedAmax ? (y > x ? y : x) : (y < x ? y : x));
  } else {
    // v replaces a when it is beyond it or NaN; a NaN a stays
    const Acc r = OP == kRedAmax ? (!(v <= a) ? v : a) : (!(v >= a) ? v : a);
    return a != a ? a : r;
  }
}
template <class T, class Acc, int OP> __device__ __forceinline__ T seg_finish(int include_self, T old, Acc acc) {
  if (include_self) acc = seg_op<T, Acc, OP>(acc, cvt<Acc>(old));
  if constexpr (std::is_integral<T>::value) return (T)acc;
  else return cvt<T>(acc);
}

// Segmented row sums over sorted (destination row, source row) pairs.  One wave owns a chunk of consecutive pairs
// (64, 128 or 256 of them: seg_chunk).  It first reads its keys and source-row ids with coalesced loads and hands them
// out with readlane, so the row loads never wait on an index load.  Rows are fetched 8 at a time with non-temporal
// loads, and together with them self's row of every run that opens in the batch, so a destination row costs no round
// trip of its own: when its run ends, sum and old row are both in registers and the new row is stored.  A bare
// row-summing loop of this shape (no run logic) moves 6.3 TB/s over 1 Mi random rows of 1 KiB whether it fetches 2, 4,
// 8 or 16 rows per round trip, with or without the next batch requested ahead, so the kernel keeps no prefetch
// registers and no LDS, and waits once per batch.  Source rows are read with non-temporal loads; self's rows are
// read and written with plain ones (they are touched twice within a few microseconds: 289 -> 282 us on 1 Mi rows
// into 64 Ki).  The few stores cost more than their bytes: with one finished run per 16 rows the loop takes 214 us
// against 168 us without them, and every wait of every wave grows alike (3.5 -> 4.0 us per batch, whether the
// batch before it stored or not) - the memory system as a whole slows down when writes are sprinkled over a read
// stream, so collecting the stores in LDS, or splitting short and long runs into two kernels, gains nothing.
// The accumulation order is fixed (fp32 for the floating dtypes), and every destination row is updated by exactly one
// wave: a run that lies inside the chunk updates self here; the pieces of a run that crosses chunk boundaries are
// parked in part_a / part_b and added by the combine kernels in chunk order.
template <class T, int VEC, int OP>
__global__ __launch_bounds__(kBlock) void seg_rows_kernel(const SegRowArgs a) {
  using Acc = typename SegAcc<T>::type;
  constexpr bool GENERAL = OP >= 0;
  const Acc ident = seg_identity<T, Acc, OP>();
  constexpr int kBatch = 8;
  constexpr int H = kMaxChunk / kWave;
  static_assert(kWave % kBatch == 0, "a batch reads its keys from one register");
  const int lane = threadIdx.x & (kWave - 1);
  const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int64_t chunk = (int64_t)blockIdx.x * kWaves + w;
  if (chunk >= a.nchunks) return;
  const int64_t j0 = chunk * a.chunk;
  const int cnt = (int)std::min<int64_t>(a.chunk, a.n - j0);
  // lane l holds entries l, 64 + l, ... of the chunk; slots past the end of the chunk repeat its last entry, so a batch
  // that straddles the end reads valid rows (and ignores them)
  // (held as 4-element vectors: an array indexed by the batch's register number is moved to LDS by the compiler)
  typedef uint32_t RegVec __attribute__((ext_vector_type(H)));
  RegVec kreg = 0u, vreg = 0u;
#pragma unroll
  for (int h = 0; h < H; ++h) {
    if (h * kWave < cnt) {
      const int64_t j = j0 + std::min(h * kWave + lane, cnt - 1);
      kreg[h] = a.keys[j];
      vreg[h] = a.vals[j];
    }
  }
  auto pick = [&](const RegVec& r, int h) -> uint32_t { return r[h]; };       // h is the same in every lane
  const uint32_t first_key = (uint32_t)__builtin_amdgcn_readlane((int)kreg[0], 0);
  const uint32_t last_key = (uint32_t)__builtin_amdgcn_readlane((int)pick(kreg, (cnt - 1) / kWave), (cnt - 1) & (kWave - 1));
  const bool from_before = j0 > 0 && a.keys[j0 - 1] == first_key;
  const bool to_after = j0 + cnt < a.n && a.keys[j0 + cnt] == last_key;
  const bool use_self = !GENERAL || a.include_self;
  Acc* const part_a = (Acc*)a.part_a;
  Acc* const part_b = (Acc*)a.part_b;
  for (int64_t cb = 0; cb < a.width; cb += kWave * VEC) {
    const int64_t col = cb + (int64_t)lane * VEC;
    const bool active = col < a.width;
    // inactive lanes re-read column 0
    const uint32_t lane_bytes = (uint32_t)((active ? col : 0) * (int64_t)sizeof(T));
    auto src_at = [&](uint32_t r) -> const T* { return (const T*)(a.src + (int64_t)r * a.src_row * (int64_t)sizeof(T) + lane_bytes); };
    auto self_at = [&](uint32_t r) -> T* { return (T*)(a.self + (int64_t)r * a.self_row * (int64_t)sizeof(T) + lane_bytes); };
    Vec<Acc, VEC> acc;
    Vec<T, VEC> held;                          // self's row of the run being summed (runs that open in this chunk)
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      acc.v[e] = ident;
      held.v[e] = T();
    }
    uint32_t cur = first_key;
    bool first_piece = true;

    // a piece of a run that crosses a chunk boundary.  (Adding integer pieces to their row with atomics instead, and
    // dropping the combine pass for integers, measured slower: the chunks of the hottest row then queue on the same
    // 256 addresses.)
    auto park = [&](Acc* part) {
      if (active) vec_store<Acc, VEC, false>(part + chunk * a.width + col, acc);      // read again soon by the combine pass
    };
    // the run of `cur` ends: continuation pieces go to part_a, whole runs to self
    auto finish = [&]() {
      if (first_piece && from_before) {
        park(part_a);
      } else if (active) {
        Vec<T, VEC> t;
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
          if constexpr (GENERAL) t.v[q] = seg_finish<T, Acc, OP>(a.include_self, held.v[q], acc.v[q]);
          else t.v[q] = seg_add<T, Acc>(held.v[q], scaled<T, Acc>(acc.v[q], a.alpha_f, a.alpha_i));
        }
        vec_store<T, VEC, false>(self_at(cur), t);
      }
    };

    for (int e0 = 0; e0 < cnt; e0 += kBatch) {
      const uint32_t kr = pick(kreg, e0 / kWave), vr = pick(vreg, e0 / kWave);
      uint32_t k[kBatch];
      bool fresh[kBatch];                      // the entry opens a run that ends in this chunk: its sum is added to self's row
      Vec<T, VEC> row[kBatch], old[kBatch];
      uint32_t prev = cur;                     // key of entry e0 - 1
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        const int l = (e0 & (kWave - 1)) + b;
        k[b] = (uint32_t)__builtin_amdgcn_readlane((int)kr, l);
        const uint32_t v = (uint32_t)__builtin_amdgcn_readlane((int)vr, l);
        row[b] = vec_load<T, VEC, true>(src_at(v));
        const bool opens = e0 + b == 0 ? !from_before : k[b] != prev;
        fresh[b] = opens && e0 + b < cnt && use_self && !(to_after && k[b] == last_key);
        old[b] = Vec<T, VEC>{};                // a defined value on the other path keeps the register allocation compact
        if (fresh[b]) old[b] = vec_load<T, VEC, false>(self_at(k[b]));
        prev = k[b];
      }
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        if (e0 + b < cnt) {
          if (k[b] != cur) {
            finish();
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc.v[q] = ident;
            cur = k[b];
            first_piece = false;
          }
          if (fresh[b]) held = old[b];
#pragma unroll
          for (int q = 0; q < VEC; ++q) {
            if constexpr (GENERAL) acc.v[q] = seg_op<T, Acc, OP>(acc.v[q], cvt<Acc>(row[b].v[q]));
            else acc.v[q] += cvt<Acc>(row[b].v[q]);
          }
        }
      }
    }
    // last piece of the chunk
    if (!(first_piece && from_before) && to_after) park(part_b);
    else finish();
  }
  if (lane == 0) {
    // first piece continues from before: END if it stops inside this chunk, THROUGH if the whole chunk is one run that goes on
    const bool single = first_key == last_key;
    a.flag_a[chunk] = from_before ? ((single && to_after) ? kThrough : kEnd) : kNone;
    const bool start = to_after && !(single && from_before);
    a.key_b[chunk] = last_key;
    if (start) a.start_list[atomicAdd(a.nstart, 1u)] = (uint32_t)chunk;
  }
}

// For every chunk that STARTS a run continuing into later chunks: add, in chunk order, the start piece and the
// continuation pieces of the following chunks, then update self once.  Nearly all such runs have one or two
// continuation pieces, and a workgroup per run spends its time in barriers and dependent loads (23 us for the 8192
// chunks of 1 Mi Zipf-distributed rows); so one WAVE takes a run, reads the flags of the next kShortRun chunks in one
// load, and adds up to kShortRun pieces with all their loads in flight together.  A longer run (a hot destination row)
// goes onto long_list for the kernel below.  The order of additions depends only on the data.
// (One kernel that does both - 16 waves per workgroup, each on a short run, then all of them on the long runs the
// workgroup met - measured 23 us against 4.9 + 11.3 us: the workgroup that meets the hottest row does its share of
// short runs first.)
template <class T, int VEC, int OP>
__global__ __launch_bounds__(kBlock) void seg_combine_kernel(const SegRowArgs a) {
  using Acc = typename SegAcc<T>::type;
  constexpr bool GENERAL = OP >= 0;
  const Acc* const part_a = (const Acc*)a.part_a;
  const Acc* const part_b = (const Acc*)a.part_b;
  const int lane = threadIdx.x & (kWave - 1);
  const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const unsigned int nstart = *a.nstart;
  const unsigned int stride = gridDim.x * kWaves;
  for (unsigned int s = blockIdx.x * kWaves + w; s < nstart; s += stride) {
    const int64_t c = a.start_list[s];
    // the run ends at the first chunk after c whose flag is not THROUGH (there is one: a THROUGH chunk has a successor)
    const int64_t i = c + 1 + lane;
    const bool stop = lane < kShortRun && i < a.nchunks && a.flag_a[i] != kThrough;
    const unsigned long long stops = __ballot(stop);
    if (stops == 0ull) {
      if (lane == 0) a.long_list[atomicAdd(a.nlong, 1u)] = (uint32_t)c;
      continue;
    }
    const int nparts = __builtin_amdgcn_readfirstlane(__builtin_ctzll(stops) + 1);      // continuation pieces c+1 .. c+nparts
    const uint32_t key = a.key_b[c];
    for (int64_t cb = 0; cb < a.width; cb += kWave * VEC) {
      const int64_t col = cb + (int64_t)lane * VEC;
      if (col >= a.width) continue;
      Vec<Acc, VEC> piece[kShortRun];
      const Vec<Acc, VEC> head = vec_load<Acc, VEC, false>(part_b + c * a.width + col);
      T* const d = (T*)a.self + (int64_t)key * a.self_row + col;
      const Vec<T, VEC> old = vec_load<T, VEC, false>(d);
      piece[0] = vec_load<Acc, VEC, false>(part_a + (c + 1) * a.width + col);
      if (nparts > 1) {
#pragma unroll
        for (int p = 1; p < kShortRun; ++p)            // clamped: the loads past the run re-read its last piece and are ignored
          piece[p] = vec_load<Acc, VEC, false>(part_a + (c + 1 + std::min(p, nparts - 1)) * a.width + col);
      }
      Vec<Acc, VEC> t = head;
#pragma unroll
      for (int p = 0; p < kShortRun; ++p)
        if (p < nparts) {
#pragma unroll
          for (int q = 0; q < VEC; ++q) {
            if constexpr (GENERAL) t.v[q] = seg_op<T, Acc, OP>(t.v[q], piece[p].v[q]);
            else t.v[q] += piece[p].v[q];
          }
        }
      Vec<T, VEC> r;
#pragma unroll
      for (int q = 0; q < VEC; ++q) {
        if constexpr (GENERAL) r.v[q] = seg_finish<T, Acc, OP>(a.include_self, old.v[q], t.v[q]);
        else r.v[q] = seg_add<T, Acc>(old.v[q], scaled<T, Acc>(t.v[q], a.alpha_f, a.alpha_i));
      }
      vec_store<T, VEC, false>(d, r);
    }
  }
}

// The runs with more than kShortRun continuation pieces: one workgroup of kLongWaves waves per run.  Its waves take
// contiguous sub-ranges of the pieces and their sums are then added in wave order.
template <class T, int VEC, int OP>
__global__ __launch_bounds__(kLongWaves * kWave) void seg_combine_long_kernel(const SegRowArgs a) {
  using Acc = typename SegAcc<T>::type;
  constexpr bool GENERAL = OP >= 0;
  const Acc ident = seg_identity<T, Acc, OP>();
  __shared__ long long end_chunk;
  __shared__ Acc sub[kLongWaves][kWave * VEC];
  const Acc* const part_a = (const Acc*)a.part_a;
  const Acc* const part_b = (const Acc*)a.part_b;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const unsigned int nlong = *a.nlong;
  for (unsigned int s = blockIdx.x; s < nlong; s += gridDim.x) {
    const int64_t c = a.long_list[s];
    if (threadIdx.x == 0) end_chunk = a.nchunks - 1;
    __syncthreads();
    // first chunk after c whose continuation piece is not THROUGH
    for (int64_t base = c + 1; base < a.nchunks; base += kLongWaves * kWave) {
      const int64_t i = base + threadIdx.x;
      const bool stop = i < a.nchunks && a.flag_a[i] != kThrough;
      const bool any = __syncthreads_or(stop);
      if (stop) atomicMin((unsigned long long*)&end_chunk, (unsigned long long)i);
      if (any) break;
    }
    __syncthreads();
    const int64_t cend = end_chunk;
    const int64_t nparts = cend - c;                       // continuation pieces c+1 .. cend
    const int64_t per = (nparts + kLongWaves - 1) / kLongWaves;
    const int64_t p0 = c + 1 + (int64_t)w * per;
    const int64_t p1 = std::min<int64_t>(p0 + per, cend + 1);
    const uint32_t key = a.key_b[c];
    for (int64_t cb = 0; cb < a.width; cb += kWave * VEC) {
      const int64_t col = cb + (int64_t)lane * VEC;
      const bool active = col < a.width;
      Acc acc[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] = ident;
      if (active) {
#pragma unroll 16
        for (int64_t p = p0; p < p1; ++p) {
          const Vec<Acc, VEC> piece = vec_load<Acc, VEC, false>(part_a + p * a.width + col);
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            if constexpr (GENERAL) acc[e] = seg_op<T, Acc, OP>(acc[e], piece.v[e]);
            else acc[e] += piece.v[e];
          }
        }
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) sub[w][lane * VEC + e] = acc[e];
      __syncthreads();
      if (w == 0 && active) {
        const Acc* b = part_b + c * a.width + col;
        T* d = (T*)a.self + (int64_t)key * a.self_row + col;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          Acc t = b[e];
          if constexpr (GENERAL) {
            for (int ww = 0; ww < kLongWaves; ++ww) t = seg_op<T, Acc, OP>(t, sub[ww][lane * VEC + e]);
            d[e] = seg_finish<T, Acc, OP>(a.include_self, d[e], t);
          } else {
            for (int ww = 0; ww < kLongWaves; ++ww) t += sub[ww][lane * VEC + e];
            d[e] = seg_add<T, Acc>(d[e], scaled<T, Acc>(t, a.alpha_f, a.alpha_i));
          }
        }
      }
      __syncthreads();
    }
  }
}

// ---------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------
// the two kernels above on n sorted entries; the three arrays hold one record per block of kBlock entries
template <class T, bool BITS = false>
void launch_seg_reduce(const uint32_t* keys, const uint32_t* vals, int64_t n, const ElemArgs& ea, int mode, int include_self,
                       char* part_a, char* part_b, char* flag_a, hipStream_t s) {
  const unsigned nb = (unsigned)((n + kBlock - 1) / kBlock);
  const RedPieces pc{part_a, part_b, (uint8_t*)flag_a};
  hipLaunchKernelGGL((seg_reduce_kernel<T, BITS>), dim3(nb), dim3(kBlock), 0, s, keys, vals, n, ea, mode, include_self, pc);
  hipLaunchKernelGGL((seg_reduce_finish_kernel<T>), dim3((nb + kBlock - 1) / kBlock), dim3(kBlock), 0, s, keys, n, (int64_t)nb, ea, mode,
                     include_self, pc);
}
inline size_t seg_reduce_blocks(int64_t n) { return (size_t)((n + kBlock - 1) / kBlock); }
bool index_dtype_ok(int dt) { return dt == TX_I32 || dt == TX_I64; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
int bits_for(uint64_t max_value) {
  int b = 1;
  while (b < 64 && (max_value >> b)) ++b;
  return b;
}

struct ScatterPlan {
  bool row_mode;
  int64_t n;            // sorted entries
  int64_t width;        // row mode: elements per row
  int passes;
  int nblocks;          // sort workgroups
  int64_t nchunks;
  int chunk;            // row mode: sorted rows per wave
  size_t off_keys[2], off_vals[2], off_hist, off_totals, off_part_a, off_part_b, off_flag_a, off_key_b, off_start_list,
      off_long_list, off_counter;
  size_t bytes;
};

// row mode: dim 0; index is a row id broadcast over the trailing dims; the trailing dims of
// index, src and self agree and are laid out contiguously in src and self
bool is_row_mode(const tx_tensor* self, int dim, const tx_tensor* index, const tx_tensor* src) {
  if (dim != 0 || self->ndim < 2) return false;
  int64_t inner = 1;
  for (int d = self->ndim - 1; d >= 1; --d) {
    if (index->sizes[d] != self->sizes[d] || index->sizes[d] != src->sizes[d]) return false;
    if (index->sizes[d] > 1 && index->strides[d] != 0) return false;
    if (self->sizes[d] > 1 && (self->strides[d] != inner || src->strides[d] != inner)) return false;
    inner *= self->sizes[d];
  }
  // (a lane's byte offset inside a row is kept in 32 bits)
  return inner >= 16 && inner * dtype_size(self->dtype) < (1ll << 32) && index->sizes[0] < (1ll << 31) && self->sizes[0] < (1ll << 32);
}

tx_status scatter_plan(const tx_tensor* self, int dim, const tx_tensor* index, const tx_tensor* src, ScatterPlan* p,
                       bool allow_rows = true) {
  memset(p, 0, sizeof(*p));
  p->row_mode = allow_rows && is_row_mode(self, dim, index, src);
  uint64_t max_key;
  if (p->row_mode) {
    p->n = index->sizes[0];
    p->width = 1;
    for (int d = 1; d < self->ndim; ++d) p->width *= self->sizes[d];
    max_key = (uint64_t)std::max<int64_t>(self->sizes[0], 1) - 1;
  } else {
    p->n = numel(index);
    uintptr_t lo, hi;
    byte_extent(self, &lo, &hi);
    const uint64_t extent = (hi - lo) / dtype_size(self->dtype);
    // positions are decoded with 32-bit magic-number divisions, which hold for dividends below 2^31
    if (p->n >= (1ll << 31) || extent >= (1ull << 32))
      return fail(TX_ERR_UNSUPPORTED, "deterministic scatter_add: 2^31 or more positions, or 2^32 or more destination elements");
    max_key = extent ? extent - 1 : 0;
  }
  p->passes = (bits_for(max_key) + 7) / 8;
  p->nblocks = (int)((p->n + kSortTile - 1) / kSortTile);
  p->chunk = seg_chunk(p->n);
  p->nchunks = p->row_mode ? (p->n + p->chunk - 1) / p->chunk : 0;
  size_t o = 0;
  for (int i = 0; i < 2; ++i) { p->off_keys[i] = o; o = align_up(o + (size_t)p->n * 4, 256); }
  for (int i = 0; i < 2; ++i) { p->off_vals[i] = o; o = align_up(o + (size_t)p->n * 4, 256); }
  p->off_hist = o; o = align_up(o + (size_t)256 * p->nblocks * 4, 256);
  p->off_totals = o; o = align_up(o + 256 * 4, 256);
  if (p->row_mode) {
    const size_t acc_size = self->dtype == TX_I64 ? 8 : 4;     // fp32 accumulators for floats, the dtype itself for integers
    p->off_part_a = o; o = align_up(o + (size_t)p->nchunks * p->width * acc_size, 256);
    p->off_part_b = o; o = align_up(o + (size_t)p->nchunks * p->width * acc_size, 256);
    p->off_flag_a = o; o = align_up(o + (size_t)p->nchunks, 256);
    p->off_key_b = o; o = align_up(o + (size_t)p->nchunks * 4, 256);
    p->off_start_list = o; o = align_up(o + (size_t)p->nchunks * 4, 256);
    p->off_long_list = o; o = align_up(o + (size_t)p->nchunks * 4, 256);
    p->off_counter = o; o += 256;
  } else {                                              // element mode: the pieces of runs that cross blocks of sorted entries
    const size_t rblocks = seg_reduce_blocks(p->n);
    p->off_part_a = o; o = align_up(o + rblocks * 16, 256);
    p->off_part_b = o; o = align_up(o + rblocks * 16, 256);
    p->off_flag_a = o; o = align_up(o + rblocks, 256);
  }
  p->bytes = o;
  return TX_OK;
}

struct Alpha {
  float f;
  int64_t i;
  int64_t wrap = 0;        // not a multiplier: the extent added to negative indices (index_put_), carried along
};

void fill_scatter_elem_args(ElemArgs* a, const tx_tensor* self, int dim, const tx_tensor* index, const tx_tensor* src,
                            Alpha alpha = Alpha{1.0f, 1}) {
  a->alpha_f = alpha.f;
  a->alpha_i = alpha.i;
  a->wrap = alpha.wrap;
  fill_dims(&a->shape, index->ndim, index->sizes);
  a->dim = dim;
  a->index_is64 = index->dtype == TX_I64;
  a->index = (const char*)index->data;
  a->src = (const char*)src->data;
  a->dst = (char*)self->data;
  for (int d = 0; d < index->ndim; ++d) {
    a->istride[d] = index->strides[d];
    a->sstride[d] = src->strides[d];
    a->dstride[d] = self->strides[d];
  }
  if (index->ndim == 0) {   // 0-dim: one element, destination offset index * 0
    a->shape.n = 0;
    a->istride[0] = a->sstride[0] = a->dstride[0] = 0;
  }
}

// first_hist_done: the caller's key kernel has already counted the first pass's histogram (row_keys_hist_kernel)
tx_status run_sort(const ScatterPlan& p, char* ws, hipStream_t s, int* result_buffer, bool first_hist_done = false) {
  uint32_t* keys[2] = {(uint32_t*)(ws + p.off_keys[0]), (uint32_t*)(ws + p.off_keys[1])};
  uint32_t* vals[2] = {(uint32_t*)(ws + p.off_vals[0]), (uint32_t*)(ws + p.off_vals[1])};
  uint32_t* hist = (uint32_t*)(ws + p.off_hist);
  uint32_t* totals = (uint32_t*)(ws + p.off_totals);
  int cur = 0;
  for (int pass = 0; pass < p.passes; ++pass) {
    const int shift = 8 * pass;
    if (pass > 0 || !first_hist_done)
      hipLaunchKernelGGL(sort_hist_kernel, dim3(p.nblocks), dim3(kBlock), 0, s, keys[cur], p.n, shift, hist, p.nblocks);
    hipLaunchKernelGGL(sort_rowscan_kernel, dim3(256), dim3(kBlock), 0, s, hist, p.nblocks, totals);
    hipLaunchKernelGGL(sort_scatter_kernel, dim3(p.nblocks), dim3(kBlock), 0, s, keys[cur], vals[cur], keys[1 - cur],
                       vals[1 - cur], p.n, shift, hist, totals, p.nblocks);
    cur = 1 - cur;
  }
  *result_buffer = cur;
  return check_launch("radix sort");
}

// Sorted scatter_add.  Floating dtypes: every index layout (row mode or element mode).  int32 / int64: row
// mode only - integer addition needs no fixed order, but grouping rows by destination replaces one atomic
// per source element by plain row sums, and hot destination rows no longer serialise on atomics.
template <class T>
tx_status scatter_deterministic(const ScatterPlan& p, const tx_tensor* self, int dim, const tx_tensor* index,
                                const tx_tensor* src, char* ws, hipStream_t s, Alpha alpha, int general_op = -1,
                                int include_self = 1) {
  constexpr int V = sizeof(T) == 2 ? 4 : 16 / sizeof(T);     // row kernels: at most 16 bytes of accumulators per lane
  constexpr int kVecBytes = V * (int)sizeof(T);
  uint32_t* keys0 = (uint32_t*)(ws + p.off_keys[0]);
  uint32_t* vals0 = (uint32_t*)(ws + p.off_vals[0]);
  ElemArgs ea;
  fill_scatter_elem_args(&ea, self, dim, index, src, alpha);
  const unsigned nb = (unsigned)((p.n + kBlock - 1) / kBlock);
  if (p.row_mode)
    hipLaunchKernelGGL(row_keys_hist_kernel, dim3(p.nblocks), dim3(kBlock), 0, s, (const char*)index->data,
                       index->dtype == TX_I64, index->strides[0], p.n, keys0, vals0, (unsigned int*)(ws + p.off_counter),
                       alpha.wrap, (uint32_t*)(ws + p.off_hist), p.nblocks);
  else
    hipLaunchKernelGGL(scatter_keys_kernel<key_value_bytes<T>()>, dim3(nb), dim3(kBlock), 0, s, ea, keys0, vals0);
  int cur;
  tx_status rc = run_sort(p, ws, s, &cur, p.row_mode && p.passes > 0);
  if (rc) return rc;
  const uint32_t* keys = (const uint32_t*)(ws + p.off_keys[cur]);
  const uint32_t* vals = (const uint32_t*)(ws + p.off_vals[cur]);
  if (!p.row_mode) {
    if constexpr (std::is_integral<T>::value) {
      return fail(TX_ERR_UNSUPPORTED, "sorted integer scatter_add needs a broadcast row index");
    } else {
      set_path("scatter-sort-elem");
      launch_seg_reduce<T, key_value_bytes<T>() != 0>(keys, vals, p.n, ea, kRedSum, 1, ws + p.off_part_a, ws + p.off_part_b, ws + p.off_flag_a, s);
      return check_launch("segmented sum");
    }
  }
  SegRowArgs a;
  a.keys = keys;
  a.vals = vals;
  a.n = p.n;
  a.nchunks = p.nchunks;
  a.chunk = p.chunk;
  a.src = (const char*)src->data;
  a.self = (char*)self->data;
  a.src_row = src->strides[0];
  a.self_row = self->strides[0];
  a.width = p.width;
  a.part_a = ws + p.off_part_a;
  a.part_b = ws + p.off_part_b;
  a.flag_a = (uint8_t*)(ws + p.off_flag_a);
  a.key_b = (uint32_t*)(ws + p.off_key_b);
  a.start_list = (uint32_t*)(ws + p.off_start_list);
  a.nstart = (unsigned int*)(ws + p.off_counter);
  a.long_list = (uint32_t*)(ws + p.off_long_list);
  a.nlong = a.nstart + 1;
  a.alpha_f = alpha.f;
  a.alpha_i = alpha.i;
  a.include_self = include_self;
  const bool al = p.width % V == 0 && (uintptr_t)src->data % kVecBytes == 0 && (uintptr_t)self->data % kVecBytes == 0 &&
                  (a.src_row * (int64_t)sizeof(T)) % kVecBytes == 0 && (a.self_row * (int64_t)sizeof(T)) % kVecBytes == 0;
  const unsigned gb = (unsigned)((p.nchunks + kWaves - 1) / kWaves);
  set_path(al ? "scatter-sort-rows" : "scatter-sort-rows-scalar");
  const unsigned cg = (unsigned)std::min<int64_t>(kCombineBlocks, (p.nchunks + kWaves - 1) / kWaves);
  const unsigned lg = (unsigned)std::min<int64_t>(kLongBlocks, p.nchunks);
  auto launch = [&](auto vec, auto op) {
    constexpr int VV = decltype(vec)::value, OP = decltype(op)::value;
    hipLaunchKernelGGL((seg_rows_kernel<T, VV, OP>), dim3(gb), dim3(kBlock), 0, s, a);
    hipLaunchKernelGGL((seg_combine_kernel<T, VV, OP>), dim3(cg), dim3(kBlock), 0, s, a);
    hipLaunchKernelGGL((seg_combine_long_kernel<T, VV, OP>), dim3(lg), dim3(kLongWaves * kWave), 0, s, a);
  };
  auto with_op = [&](auto op) {
    if (al) launch(std::integral_constant<int, V>{}, op);
    else launch(std::integral_constant<int, 1>{}, op);
  };
  if (general_op >= 0) set_path(al ? "scatter-reduce-rows" : "scatter-reduce-rows-scalar");
  if (general_op == kRedSum) with_op(std::integral_constant<int, kRedSum>{});
  else if (general_op == kRedAmax) with_op(std::integral_constant<int, kRedAmax>{});
  else if (general_op == kRedAmin) with_op(std::integral_constant<int, kRedAmin>{});
  else with_op(std::integral_constant<int, -1>{});
  return check_launch("segmented row sum");
}

tx_status scatter_checks(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* src, int* d) {
  tx_status rc;
  if ((rc = check_tensor(self, "self")) || (rc = check_tensor(index, "index")) || (rc = check_tensor(src, "src")))
    return rc;
  if (!index_dtype_ok(index->dtype)) return fail(TX_ERR_DTYPE, "index must be int32 or int64");
  if (self->dtype != src->dtype) return fail(TX_ERR_DTYPE, "scatter_add_: self and src dtypes differ");
  if (index->ndim != self->ndim || src->ndim != self->ndim)
    return fail(TX_ERR_SHAPE, "scatter_add_: self, index and src must have the same rank");
  if ((rc = wrap_dim(dim, self->ndim, d))) return rc;
  for (int i = 0; i < self->ndim; ++i) {
    if (index->sizes[i] > src->sizes[i]) return fail(TX_ERR_SHAPE, "scatter_add_: index larger than src in dim %d", i);
    if (i != *d && index->sizes[i] > self->sizes[i])
      return fail(TX_ERR_SHAPE, "scatter_add_: index larger than self in dim %d", i);
  }
  if (!no_internal_overlap(self)) return fail(TX_ERR_OVERLAP, "self has overlapping elements");
  if (partial_overlap(self, src) || partial_overlap(self, index) || (self->data == src->data && numel(src) && numel(self)))
    return fail(TX_ERR_OVERLAP, "self overlaps src or index");
  return TX_OK;
}

// shared by scatter_add_ and index_add_ (whose index is presented as a broadcast view): workspace size and dispatch
size_t scatter_ws_bytes(const tx_tensor* self, int d, const tx_tensor* index, const tx_tensor* src, int deterministic) {
  if (numel(index) == 0) return 0;
  const bool int_rows = (self->dtype == TX_I32 || self->dtype == TX_I64) && is_row_mode(self, d, index, src) &&
                        index->sizes[0] >= kIntRowModeMin;
  if (!dtype_is_float(self->dtype) && !int_rows) return 0;
  if (!deterministic && self->dtype == TX_F32) return 0;
  ScatterPlan p;
  if (scatter_plan(self, d, index, src, &p)) return 0;
  return p.bytes;
}

tx_status scatter_core(const char* name, const tx_tensor* self, int d, const tx_tensor* index, const tx_tensor* src, Alpha alpha,
                       int deterministic, void* ws, size_t ws_bytes, hipStream_t s) {
  tx_status rc;
  const int64_t n = numel(index);
  if (n == 0) return TX_OK;
  // fp16 / bf16 always take the sorted path: 16-bit atomics would round every partial sum to the half type
  if (dtype_is_float(self->dtype) && (deterministic || self->dtype != TX_F32)) {
    ScatterPlan p;
    if ((rc = scatter_plan(self, d, index, src, &p))) return rc;
    if (!ws || ws_bytes < p.bytes) return fail(TX_ERR_WORKSPACE, "%s needs %zu workspace bytes, got %zu", name, p.bytes, ws_bytes);
    if ((uintptr_t)ws % 16) return fail(TX_ERR_WORKSPACE, "%s workspace must be 16-byte aligned", name);
    switch (self->dtype) {
      case TX_F32: return scatter_deterministic<float>(p, self, d, index, src, (char*)ws, s, alpha);
      case TX_BF16: return scatter_deterministic<bf16>(p, self, d, index, src, (char*)ws, s, alpha);
      default: return scatter_deterministic<f16>(p, self, d, index, src, (char*)ws, s, alpha);
    }
  }
  // int32 / int64 with a broadcast row index: group rows by destination first and add whole rows.
  // Needs the workspace; without it (or for small inputs) fall through to one atomic per element.
  if ((self->dtype == TX_I32 || self->dtype == TX_I64) && is_row_mode(self, d, index, src) &&
      index->sizes[0] >= kIntRowModeMin && strcmp(forced_path(), "scatter-atomic") != 0) {
    ScatterPlan p;
    if (!scatter_plan(self, d, index, src, &p) && ws && ws_bytes >= p.bytes && (uintptr_t)ws % 16 == 0) {
      if (self->dtype == TX_I32) return scatter_deterministic<int32_t>(p, self, d, index, src, (char*)ws, s, alpha);
      return scatter_deterministic<int64_t>(p, self, d, index, src, (char*)ws, s, alpha);
    }
  }
  if (n >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "%s: more than 2^31 index elements", name);
  ElemArgs a;
  fill_scatter_elem_args(&a, self, d, index, src, alpha);
  const dim3 grid((unsigned)((n + kBlock - 1) / kBlock));
  set_path("scatter-atomic");
  switch (self->dtype) {
    case TX_BOOL: hipLaunchKernelGGL((scatter_add_atomic_kernel<uint8_t>), grid, dim3(kBlock), 0, s, a); break;
    case TX_I32: hipLaunchKernelGGL((scatter_add_atomic_kernel<int32_t>), grid, dim3(kBlock), 0, s, a); break;
    case TX_I64: hipLaunchKernelGGL((scatter_add_atomic_kernel<int64_t>), grid, dim3(kBlock), 0, s, a); break;
    default: hipLaunchKernelGGL((scatter_add_atomic_kernel<float>), grid, dim3(kBlock), 0, s, a); break;
  }
  return check_launch("scatter_add atomic kernel");
}

// sort plan for n (key, position) pairs whose keys are element offsets inside `self`
tx_status elem_sort_plan(const char* name, const tx_tensor* self, int64_t n, ScatterPlan* p) {
  memset(p, 0, sizeof(*p));
  p->n = n;
  uintptr_t lo, hi;
  byte_extent(self, &lo, &hi);
  const uint64_t extent = (hi - lo) / dtype_size(self->dtype);
  if (n >= (1ll << 31) || extent >= (1ull << 32))       // positions are decoded with 32-bit magic-number divisions (dividends below 2^31)
    return fail(TX_ERR_UNSUPPORTED, "%s: 2^31 or more positions, or 2^32 or more destination elements", name);
  p->passes = (bits_for(extent ? extent - 1 : 0) + 7) / 8;
  p->nblocks = (int)((n + kSortTile - 1) / kSortTile);
  size_t o = 0;
  for (int i = 0; i < 2; ++i) { p->off_keys[i] = o; o = align_up(o + (size_t)n * 4, 256); }
  for (int i = 0; i < 2; ++i) { p->off_vals[i] = o; o = align_up(o + (size_t)n * 4, 256); }
  p->off_hist = o; o = align_up(o + (size_t)256 * p->nblocks * 4, 256);
  p->off_totals = o; o = align_up(o + 256 * 4, 256);
  // the pieces of runs that cross blocks of kBlock sorted entries (scatter_reduce_): two 16-byte records and a mark per block
  const size_t rblocks = seg_reduce_blocks(n);
  p->off_part_a = o; o = align_up(o + rblocks * 16, 256);
  p->off_part_b = o; o = align_up(o + rblocks * 16, 256);
  p->off_flag_a = o; o = align_up(o + rblocks, 256);
  p->bytes = o;
  return TX_OK;
}

tx_status sort_ws_checks(const char* name, const ScatterPlan& p, void* ws, size_t ws_bytes) {
  if (!ws || ws_bytes < p.bytes) return fail(TX_ERR_WORKSPACE, "%s needs %zu workspace bytes, got %zu", name, p.bytes, ws_bytes);
  if ((uintptr_t)ws % 16) return fail(TX_ERR_WORKSPACE, "%s workspace must be 16-byte aligned", name);
  return TX_OK;
}

template <class T>
tx_status scatter_reduce_typed(const ScatterPlan& p, const tx_tensor* self, int d, const tx_tensor* index, const tx_tensor* src,
                               int mode, int include_self, char* ws, hipStream_t s) {
  ElemArgs ea;
  fill_scatter_elem_args(&ea, self, d, index, src);
  const unsigned nb = (unsigned)((p.n + kBlock - 1) / kBlock);
  hipLaunchKernelGGL(scatter_keys_kernel<key_value_bytes<T>()>, dim3(nb), dim3(kBlock), 0, s, ea, (uint32_t*)(ws + p.off_keys[0]),
                     (uint32_t*)(ws + p.off_vals[0]));
  int cur;
  tx_status rc = run_sort(p, ws, s, &cur);
  if (rc) return rc;
  set_path("scatter-reduce-sort");
  launch_seg_reduce<T, key_value_bytes<T>() != 0>((const uint32_t*)(ws + p.off_keys[cur]), (const uint32_t*)(ws + p.off_vals[cur]), p.n, ea, mode,
                                                  include_self,
                       ws + p.off_part_a, ws + p.off_part_b, ws + p.off_flag_a, s);
  return check_launch("scatter_reduce segmented kernels");
}

// scatter_reduce_ through the whole-row kernels: sum, amax, amin (an fp32 accumulator is exact for the extrema and
// inside the tolerance for sums; products and means are left to the element path), row layout, not bool
bool scatter_reduce_rows_ok(const tx_tensor* self, int d, const tx_tensor* index, const tx_tensor* src, int reduce) {
  if (reduce != TX_SCATTER_SUM && reduce != TX_SCATTER_AMAX && reduce != TX_SCATTER_AMIN) return false;
  if (self->dtype == TX_BOOL || !strcmp(forced_path(), "scatter-reduce-sort")) return false;
  return is_row_mode(self, d, index, src);
}

// index_put_: checks; fills the kernel arguments (shape I + rest, strides of every operand over it)
tx_status index_put_checks(const tx_tensor* self, const tx_tensor* const* indices, int32_t nidx, const tx_tensor* values,
                           PutArgs* a) {
  tx_status rc;
  if ((rc = check_tensor(self, "self")) || (rc = check_tensor(values, "values"))) return rc;
  if (nidx < 1 || nidx > self->ndim) return fail(TX_ERR_DIM, "index_put_: %d index tensors for a %d-dim tensor", nidx, self->ndim);
  if (!indices) return fail(TX_ERR_NULL, "index_put_: null index list");
  for (int j = 0; j < nidx; ++j) {
    if ((rc = check_tensor(indices[j], "index"))) return rc;
    if (!index_dtype_ok(indices[j]->dtype)) return fail(TX_ERR_DTYPE, "index must be int32 or int64");
  }
  if (values->dtype != self->dtype) return fail(TX_ERR_DTYPE, "index_put_: values must have self's dtype");
  int ind;
  int64_t ishape[TX_MAX_DIMS];
  if ((rc = broadcast_shapes(indices, nidx, &ind, ishape))) return rc;
  const int rest = self->ndim - nidx;
  if (ind + rest > TX_MAX_DIMS) return fail(TX_ERR_NDIM, "index_put_: index shape plus remaining dims exceed %d dims", TX_MAX_DIMS);
  int64_t vshape[TX_MAX_DIMS];
  const int vnd = ind + rest;
  for (int d = 0; d < ind; ++d) vshape[d] = ishape[d];
  for (int d = 0; d < rest; ++d) vshape[ind + d] = self->sizes[nidx + d];
  if (values->ndim > vnd) return fail(TX_ERR_SHAPE, "index_put_: values has too many dims");
  for (int d = 0; d < values->ndim; ++d) {
    const int64_t vs = values->sizes[d], ts = vshape[vnd - values->ndim + d];
    if (vs != ts && vs != 1) return fail(TX_ERR_SHAPE, "index_put_: values does not broadcast to the indexed shape");
  }
  if (!no_internal_overlap(self)) return fail(TX_ERR_OVERLAP, "self has overlapping elements");
  if (partial_overlap(self, values) || (self->data == values->data && numel(values) && numel(self)))
    return fail(TX_ERR_OVERLAP, "self overlaps values");
  for (int j = 0; j < nidx; ++j)
    if (partial_overlap(self, indices[j])) return fail(TX_ERR_OVERLAP, "self overlaps an index");
  memset(a, 0, sizeof(*a));
  fill_dims(&a->shape, vnd, vshape);
  a->nidx = nidx;
  a->ind = ind;
  for (int j = 0; j < nidx; ++j) {
    const tx_tensor* ix = indices[j];
    a->index[j] = (const char*)ix->data;
    a->is64[j] = ix->dtype == TX_I64;
    for (int d = 0; d < ix->ndim; ++d) a->istride[j][ind - ix->ndim + d] = ix->sizes[d] != 1 ? ix->strides[d] : 0;
    a->extent[j] = self->sizes[j];
    a->dstride_idx[j] = self->strides[j];
  }
  for (int d = 0; d < rest; ++d) a->dstride[ind + d] = self->strides[nidx + d];
  for (int d = 0; d < values->ndim; ++d) a->vstride[vnd - values->ndim + d] = values->sizes[d] != 1 ? values->strides[d] : 0;
  a->src = (const char*)values->data;
  a->dst = (char*)self->data;
  return TX_OK;
}

// one 1-D index tensor over dim 0 and values of exactly the shape [n, self.shape[1:]]: accumulation is scatter_add_ with
// the index broadcast over the trailing dims (whole-row sorted path); `view` is that broadcast index
bool index_put_as_rows(const tx_tensor* self, const tx_tensor* const* indices, int32_t nidx, const tx_tensor* values,
                       tx_tensor* view) {
  if (nidx != 1 || indices[0]->ndim != 1 || values->ndim != self->ndim || self->dtype == TX_BOOL) return false;
  if (values->sizes[0] != indices[0]->sizes[0]) return false;
  for (int d = 1; d < self->ndim; ++d)
    if (values->sizes[d] != self->sizes[d]) return false;
  view->data = indices[0]->data;
  view->dtype = indices[0]->dtype;
  view->ndim = self->ndim;
  for (int d = 0; d < self->ndim; ++d) {
    view->sizes[d] = values->sizes[d];
    view->strides[d] = d == 0 ? indices[0]->strides[0] : 0;
  }
  return true;
}

// index_add_: checks, and the 1-D index presented as a view of source's shape (stride 0 off `dim`)
tx_status index_add_checks(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* source, int alpha_is_int,
                           int* d, tx_tensor* view) {
  tx_status rc;
  if ((rc = check_tensor(self, "self")) || (rc = check_tensor(index, "index")) || (rc = check_tensor(source, "source")))
    return rc;
  if (!index_dtype_ok(index->dtype)) return fail(TX_ERR_DTYPE, "index must be int32 or int64");
  if (self->dtype != source->dtype) return fail(TX_ERR_DTYPE, "index_add_: self and source dtypes differ");
  if (index->ndim > 1) return fail(TX_ERR_SHAPE, "index_add_: index must be 1-D or 0-dim");
  if (source->ndim != self->ndim) return fail(TX_ERR_SHAPE, "index_add_: self and source must have the same rank");
  if ((rc = wrap_dim(dim, self->ndim, d))) return rc;
  if ((self->ndim ? source->sizes[*d] : 1) != numel(index))
    return fail(TX_ERR_SHAPE, "index_add_: source.size(dim) must be the number of indices");
  for (int i = 0; i < self->ndim; ++i)
    if (i != *d && source->sizes[i] != self->sizes[i]) return fail(TX_ERR_SHAPE, "index_add_: source and self differ in dim %d", i);
  if (!dtype_is_float(self->dtype) && !alpha_is_int) return fail(TX_ERR_SCALAR, "floating alpha with an integer / bool result");
  if (!no_internal_overlap(self)) return fail(TX_ERR_OVERLAP, "self has overlapping elements");
  if (partial_overlap(self, source) || partial_overlap(self, index) || (self->data == source->data && numel(source) && numel(self)))
    return fail(TX_ERR_OVERLAP, "self overlaps source or index");
  view->data = index->data;
  view->dtype = index->dtype;
  view->ndim = source->ndim;
  for (int i = 0; i < source->ndim; ++i) {
    view->sizes[i] = source->sizes[i];
    view->strides[i] = i == *d ? (index->ndim ? index->strides[0] : 0) : 0;
  }
  return TX_OK;
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

tx_status tx_gather(const tx_tensor* out, const tx_tensor* src, int64_t dim, const tx_tensor* index, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(src, "src")) || (rc = check_tensor(index, "index"))) return rc;
  if (!index_dtype_ok(index->dtype)) return fail(TX_ERR_DTYPE, "index must be int32 or int64");
  if (out->dtype != src->dtype) return fail(TX_ERR_DTYPE, "gather: out must have src's dtype");
  // ranks must agree, a 0-dim tensor counting as 1-D with one element
  if (std::max(index->ndim, 1) != std::max(src->ndim, 1)) return fail(TX_ERR_SHAPE, "gather: index and src must have the same rank");
  int d;
  if ((rc = wrap_dim(dim, src->ndim, &d))) return rc;
  for (int i = 0; i < src->ndim && index->ndim; ++i)
    if (i != d && index->sizes[i] > src->sizes[i]) return fail(TX_ERR_SHAPE, "gather: index larger than src in dim %d", i);
  if (!same_sizes(out, index->ndim, index->sizes)) return fail(TX_ERR_SHAPE, "gather: out must have index's shape");
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  if (partial_overlap(out, src) || partial_overlap(out, index) || (out->data == src->data && numel(out) && numel(src)))
    return fail(TX_ERR_OVERLAP, "out overlaps src or index");
  set_path("");
  const int64_t n = numel(out);
  if (n == 0) return TX_OK;
  if (n >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "gather: more than 2^31 output elements");
  if (index_validation_on() &&
      (rc = validate_index(index, 0, src->ndim ? src->sizes[d] : 1, "gather", as_stream(stream)))) return rc;
  ElemArgs a;
  memset(&a, 0, sizeof(a));
  fill_dims(&a.shape, index->ndim, index->sizes);
  a.dim = src->ndim ? d : 0;
  a.index_is64 = index->dtype == TX_I64;
  a.index = (const char*)index->data;
  a.src = (const char*)src->data;
  a.dst = (char*)out->data;
  for (int i = 0; i < index->ndim; ++i) {
    a.istride[i] = index->strides[i];
    a.sstride[i] = i < src->ndim ? src->strides[i] : 0;      // 0-dim src read through a 1-D index: one element
    a.dstride[i] = out->strides[i];
  }
  if (index->ndim == 0) a.sstride[0] = a.istride[0] = a.dstride[0] = 0;
  const dim3 grid((unsigned)((n + kBlock * kGatherU - 1) / (kBlock * kGatherU)));
  hipStream_t s = as_stream(stream);
  set_path("gather");
  switch (dtype_size(src->dtype)) {
    case 1: hipLaunchKernelGGL((gather_kernel<uint8_t>), grid, dim3(kBlock), 0, s, a, 0); break;
    case 2: hipLaunchKernelGGL((gather_kernel<uint16_t>), grid, dim3(kBlock), 0, s, a, 0); break;
    case 4: hipLaunchKernelGGL((gather_kernel<uint32_t>), grid, dim3(kBlock), 0, s, a, 0); break;
    default: hipLaunchKernelGGL((gather_kernel<uint64_t>), grid, dim3(kBlock), 0, s, a, 0); break;
  }
  return check_launch("gather kernel");
}

tx_status tx_index_select(const tx_tensor* out, const tx_tensor* src, int64_t dim, const tx_tensor* index,
                          void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(src, "src")) || (rc = check_tensor(index, "index"))) return rc;
  if (!index_dtype_ok(index->dtype)) return fail(TX_ERR_DTYPE, "index must be int32 or int64");
  if (out->dtype != src->dtype) return fail(TX_ERR_DTYPE, "index_select: out must have src's dtype");
  if (index->ndim > 1) return fail(TX_ERR_SHAPE, "index_select: index must be 1-D or 0-dim");
  int d;
  if ((rc = wrap_dim(dim, src->ndim, &d))) return rc;
  const int64_t nsel = index->ndim ? index->sizes[0] : 1;
  const int64_t istride = index->ndim ? index->strides[0] : 0;
  if (src->ndim == 0) {
    if (nsel != 1 || out->ndim != 0) return fail(TX_ERR_SHAPE, "index_select on a 0-dim src takes one index");
  } else {
    if (out->ndim != src->ndim) return fail(TX_ERR_SHAPE, "index_select: out rank");
    for (int i = 0; i < src->ndim; ++i)
      if (out->sizes[i] != (i == d ? nsel : src->sizes[i])) return fail(TX_ERR_SHAPE, "index_select: out shape");
  }
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  if (partial_overlap(out, src) || partial_overlap(out, index) || (out->data == src->data && numel(out) && numel(src)))
    return fail(TX_ERR_OVERLAP, "out overlaps src or index");
  set_path("");
  const int64_t n = numel(out);
  if (n == 0) return TX_OK;
  hipStream_t s = as_stream(stream);
  if (index_validation_on() && (rc = validate_index(index, 0, src->ndim ? src->sizes[d] : 1, "index_select", s))) return rc;
  const int es = dtype_size(src->dtype);
  // fast path: dims below `dim` form one contiguous run in src and out; dims above collapse to one stride
  if (src->ndim >= 1) {
    int64_t inner = 1;
    bool ok = true;
    for (int i = src->ndim - 1; i > d; --i) {
      if (src->sizes[i] > 1 && (src->strides[i] != inner || out->strides[i] != inner)) ok = false;
      inner *= src->sizes[i];
    }
    int64_t outer = 1, so = 0, oo = 0;
    for (int i = d - 1; i >= 0; --i) {
      if (src->sizes[i] > 1) {
        if (outer == 1) { so = src->strides[i]; oo = out->strides[i]; }
        else if (src->strides[i] != so * outer || out->strides[i] != oo * outer) ok = false;
      }
      outer *= src->sizes[i];
    }
    const int64_t bytes = inner * es;
    ok = ok && bytes >= 64 && bytes % 16 == 0 && (uintptr_t)src->data % 16 == 0 && (uintptr_t)out->data % 16 == 0 &&
         (src->strides[d] * es) % 16 == 0 && (out->strides[d] * es) % 16 == 0 && (so * es) % 16 == 0 && (oo * es) % 16 == 0 &&
         outer * nsel < (1ll << 31);
    if (ok) {
      RowCopyArgs a;
      a.index = (const char*)index->data;
      a.src = (const char*)src->data;
      a.dst = (char*)out->data;
      a.index_is64 = index->dtype == TX_I64;
      a.istride = istride;
      a.nsel = nsel;
      a.nsel_div = FastDiv((uint32_t)nsel);
      a.rows = outer * nsel;
      a.src_outer = so * es;
      a.dst_outer = oo * es;
      a.src_dim = src->strides[d] * es;
      a.dst_dim = out->strides[d] * es;
      a.vecs = bytes / 16;
      const int64_t waves = (a.rows + kRowsPerWave - 1) / kRowsPerWave;
      set_path("index-select-rows");
      hipLaunchKernelGGL(index_select_rows_kernel, dim3((unsigned)((waves + kBlock / kWave - 1) / (kBlock / kWave))), dim3(kBlock), 0, s, a);
      return check_launch("index_select row kernel");
    }
  }
  if (n >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "index_select: more than 2^31 elements on the generic path");
  ElemArgs a;
  fill_dims(&a.shape, out->ndim, out->sizes);
  a.dim = d;
  a.index_is64 = index->dtype == TX_I64;
  a.index = (const char*)index->data;
  a.src = (const char*)src->data;
  a.dst = (char*)out->data;
  for (int i = 0; i < out->ndim; ++i) {
    a.istride[i] = 0;
    a.sstride[i] = src->strides[i];
    a.dstride[i] = out->strides[i];
  }
  a.istride[d] = istride;
  if (out->ndim == 0) { a.dim = 0; a.sstride[0] = a.dstride[0] = a.istride[0] = 0; }
  const dim3 grid((unsigned)((n + kBlock * kGatherU - 1) / (kBlock * kGatherU)));
  set_path("index-select-generic");
  switch (es) {
    case 1: hipLaunchKernelGGL((gather_kernel<uint8_t>), grid, dim3(kBlock), 0, s, a, 1); break;
    case 2: hipLaunchKernelGGL((gather_kernel<uint16_t>), grid, dim3(kBlock), 0, s, a, 1); break;
    case 4: hipLaunchKernelGGL((gather_kernel<uint32_t>), grid, dim3(kBlock), 0, s, a, 1); break;
    default: hipLaunchKernelGGL((gather_kernel<uint64_t>), grid, dim3(kBlock), 0, s, a, 1); break;
  }
  return check_launch("index_select generic kernel");
}

size_t tx_scatter_add_workspace_bytes(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* src,
                                      int deterministic) {
  int d;
  if (scatter_checks(self, dim, index, src, &d)) return 0;
  return scatter_ws_bytes(self, d, index, src, deterministic);
}

tx_status tx_scatter_add_(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* src,
                          int deterministic, void* ws, size_t ws_bytes, void* stream) {
  int d;
  tx_status rc = scatter_checks(self, dim, index, src, &d);
  if (rc) return rc;
  set_path("");
  if (index_validation_on() && numel(index) &&
      (rc = validate_index(index, 0, self->ndim ? self->sizes[d] : 1, "scatter_add_", as_stream(stream)))) return rc;
  return scatter_core("scatter_add_", self, d, index, src, Alpha{1.0f, 1}, deterministic, ws, ws_bytes, as_stream(stream));
}

size_t tx_scatter_reduce_workspace_bytes(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* src,
                                         int reduce, int include_self) {
  int d;
  if (scatter_checks(self, dim, index, src, &d) || numel(index) == 0) return 0;
  if (reduce == TX_SCATTER_SUM && include_self) return scatter_ws_bytes(self, d, index, src, 1);
  ScatterPlan p;
  if (scatter_reduce_rows_ok(self, d, index, src, reduce)) return scatter_plan(self, d, index, src, &p) ? 0 : p.bytes;
  if (elem_sort_plan("scatter_reduce_", self, numel(index), &p)) return 0;
  return p.bytes;
}

tx_status tx_scatter_reduce_(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* src, int reduce,
                             int include_self, void* ws, size_t ws_bytes, void* stream) {
  int d;
  tx_status rc = scatter_checks(self, dim, index, src, &d);
  if (rc) return rc;
  if (reduce < TX_SCATTER_SUM || reduce > TX_SCATTER_AMIN) return fail(TX_ERR_SCALAR, "scatter_reduce_: unknown reduction %d", reduce);
  if (self->dtype == TX_BOOL && reduce == TX_SCATTER_MEAN) return fail(TX_ERR_DTYPE, "scatter_reduce_: no mean of bools");
  set_path("");
  const int64_t n = numel(index);
  if (n == 0) return TX_OK;
  hipStream_t s = as_stream(stream);
  if (index_validation_on() && (rc = validate_index(index, 0, self->ndim ? self->sizes[d] : 1, "scatter_reduce_", s))) return rc;
  // a sum that keeps self is scatter_add_ (sorted, so that it is reproducible)
  if (reduce == TX_SCATTER_SUM && include_self)
    return scatter_core("scatter_reduce_", self, d, index, src, Alpha{1.0f, 1}, 1, ws, ws_bytes, s);
  ScatterPlan p;
  if (scatter_reduce_rows_ok(self, d, index, src, reduce)) {
    // a row id broadcast over the trailing dims: whole rows, sorted by destination, as scatter_add_ does
    if ((rc = scatter_plan(self, d, index, src, &p)) || (rc = sort_ws_checks("scatter_reduce_", p, ws, ws_bytes))) return rc;
    const Alpha one{1.0f, 1};
    switch (self->dtype) {
      case TX_F32: return scatter_deterministic<float>(p, self, d, index, src, (char*)ws, s, one, reduce, include_self);
      case TX_BF16: return scatter_deterministic<bf16>(p, self, d, index, src, (char*)ws, s, one, reduce, include_self);
      case TX_F16: return scatter_deterministic<f16>(p, self, d, index, src, (char*)ws, s, one, reduce, include_self);
      case TX_I32: return scatter_deterministic<int32_t>(p, self, d, index, src, (char*)ws, s, one, reduce, include_self);
      default: return scatter_deterministic<int64_t>(p, self, d, index, src, (char*)ws, s, one, reduce, include_self);
    }
  }
  if ((rc = elem_sort_plan("scatter_reduce_", self, n, &p)) || (rc = sort_ws_checks("scatter_reduce_", p, ws, ws_bytes))) return rc;
  switch (self->dtype) {
    case TX_F32: return scatter_reduce_typed<float>(p, self, d, index, src, reduce, include_self, (char*)ws, s);
    case TX_BF16: return scatter_reduce_typed<bf16>(p, self, d, index, src, reduce, include_self, (char*)ws, s);
    case TX_F16: return scatter_reduce_typed<f16>(p, self, d, index, src, reduce, include_self, (char*)ws, s);
    case TX_I32: return scatter_reduce_typed<int32_t>(p, self, d, index, src, reduce, include_self, (char*)ws, s);
    case TX_BOOL: return scatter_reduce_typed<uint8_t>(p, self, d, index, src, reduce, include_self, (char*)ws, s);
    default: return scatter_reduce_typed<int64_t>(p, self, d, index, src, reduce, include_self, (char*)ws, s);
  }
}

size_t tx_index_put_workspace_bytes(const tx_tensor* self, const tx_tensor* const* indices, int32_t nidx,
                                    const tx_tensor* values, int accumulate) {
  PutArgs a;
  if (index_put_checks(self, indices, nidx, values, &a)) return 0;
  tx_tensor view;
  if (accumulate && index_put_as_rows(self, indices, nidx, values, &view)) return scatter_ws_bytes(self, 0, &view, values, 1);
  if (!accumulate || !dtype_is_float(self->dtype) || a.shape.numel == 0) return 0;
  ScatterPlan p;
  if (elem_sort_plan("index_put_", self, a.shape.numel, &p)) return 0;
  return p.bytes;
}

tx_status tx_index_put_(const tx_tensor* self, const tx_tensor* const* indices, int32_t nidx, const tx_tensor* values,
                        int accumulate, void* ws, size_t ws_bytes, void* stream) {
  PutArgs a;
  tx_status rc = index_put_checks(self, indices, nidx, values, &a);
  if (rc) return rc;
  set_path("");
  const int64_t n = a.shape.numel;
  if (n == 0) return TX_OK;
  if (n >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "index_put_: more than 2^31 value elements");
  hipStream_t s = as_stream(stream);
  if (index_validation_on())
    for (int j = 0; j < nidx; ++j)                          // negative indices wrap once: [-size, size)
      if ((rc = validate_index(indices[j], -self->sizes[j], self->sizes[j], "index_put_", s))) return rc;
  tx_tensor view;
  if (accumulate && index_put_as_rows(self, indices, nidx, values, &view))
    return scatter_core("index_put_", self, 0, &view, values, Alpha{1.0f, 1, self->sizes[0]}, 1, ws, ws_bytes, s);
  const dim3 grid((unsigned)((n + kBlock - 1) / kBlock));
  if (!accumulate && index_put_as_rows(self, indices, nidx, values, &view) && self->ndim >= 2 && strcmp(forced_path(), "index-put") != 0) {
    // whole rows: trailing dims dense in both tensors, rows of whole 16-byte vectors at 16-byte-aligned addresses
    const int es = dtype_size(self->dtype);
    int64_t row_elems = 1;
    bool dense = true;
    for (int d = self->ndim - 1; d >= 1; --d) {
      if (self->sizes[d] != 1 && (self->strides[d] != row_elems || values->strides[d] != row_elems)) dense = false;
      row_elems *= self->sizes[d];
    }
    const int64_t row_bytes = row_elems * es;
    if (dense && row_bytes > 0 && row_bytes % 16 == 0 && (uintptr_t)self->data % 16 == 0 && (uintptr_t)values->data % 16 == 0 &&
        (self->strides[0] * es) % 16 == 0 && (values->strides[0] * es) % 16 == 0 && self->strides[0] >= 0 && values->sizes[0] < (1ll << 31)) {
      RowPutArgs r;
      r.index = (const char*)indices[0]->data;
      r.index_is64 = indices[0]->dtype == TX_I64;
      r.istride = indices[0]->strides[0];
      r.src = (const char*)values->data;
      r.dst = (char*)self->data;
      r.rows = values->sizes[0];
      r.extent = self->sizes[0];
      r.src_row = values->strides[0] * es;
      r.dst_row = self->strides[0] * es;
      r.vecs = row_bytes / 16;
      const int64_t waves = (r.rows + kRowsPerWave - 1) / kRowsPerWave;
      const int64_t blocks = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
      set_path("index-put-rows");
      hipLaunchKernelGGL(index_put_rows_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, r);
      return check_launch("index_put row kernel");
    }
  }
  if (!accumulate) {
    set_path("index-put");
    switch (dtype_size(self->dtype)) {
      case 1: hipLaunchKernelGGL((index_put_kernel<uint8_t, 0>), grid, dim3(kBlock), 0, s, a); break;
      case 2: hipLaunchKernelGGL((index_put_kernel<uint16_t, 0>), grid, dim3(kBlock), 0, s, a); break;
      case 4: hipLaunchKernelGGL((index_put_kernel<uint32_t, 0>), grid, dim3(kBlock), 0, s, a); break;
      default: hipLaunchKernelGGL((index_put_kernel<uint64_t, 0>), grid, dim3(kBlock), 0, s, a); break;
    }
    return check_launch("index_put kernel");
  }
  if (!dtype_is_float(self->dtype)) {
    set_path("index-put-atomic");
    switch (self->dtype) {
      case TX_BOOL: hipLaunchKernelGGL((index_put_kernel<uint8_t, 1>), grid, dim3(kBlock), 0, s, a); break;
      case TX_I32: hipLaunchKernelGGL((index_put_kernel<int32_t, 1>), grid, dim3(kBlock), 0, s, a); break;
      default: hipLaunchKernelGGL((index_put_kernel<int64_t, 1>), grid, dim3(kBlock), 0, s, a); break;
    }
    return check_launch("index_put atomic kernel");
  }
  // floats: destination offsets as sort keys, then each run summed in position order (binary64) by its first entry
  ScatterPlan p;
  if ((rc = elem_sort_plan("index_put_", self, n, &p)) || (rc = sort_ws_checks("index_put_", p, ws, ws_bytes))) return rc;
  char* w = (char*)ws;
  a.keys = (uint32_t*)(w + p.off_keys[0]);
  a.vals = (uint32_t*)(w + p.off_vals[0]);
  hipLaunchKernelGGL((index_put_kernel<uint8_t, 2>), grid, dim3(kBlock), 0, s, a);
  int cur;
  if ((rc = run_sort(p, w, s, &cur))) return rc;
  // the segmented sum maps a position back to its value through the value shape and strides
  ElemArgs ea;
  memset(&ea, 0, sizeof(ea));
  ea.shape = a.shape;
  for (int d = 0; d < a.shape.n; ++d) ea.sstride[d] = a.vstride[d];
  ea.src = a.src;
  ea.dst = a.dst;
  ea.alpha_f = 1.0f;
  ea.alpha_i = 1;
  set_path("index-put-sort");
  const uint32_t* keys = (const uint32_t*)(w + p.off_keys[cur]);
  const uint32_t* vals = (const uint32_t*)(w + p.off_vals[cur]);
  char* pa = w + p.off_part_a;
  char* pb = w + p.off_part_b;
  char* fa = w + p.off_flag_a;
  switch (self->dtype) {
    case TX_F32: launch_seg_reduce<float>(keys, vals, n, ea, kRedSum, 1, pa, pb, fa, s); break;
    case TX_BF16: launch_seg_reduce<bf16>(keys, vals, n, ea, kRedSum, 1, pa, pb, fa, s); break;
    default: launch_seg_reduce<f16>(keys, vals, n, ea, kRedSum, 1, pa, pb, fa, s); break;
  }
  return check_launch("index_put segmented sum");
}

size_t tx_index_add_workspace_bytes(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* source,
                                    int deterministic) {
  int d;
  tx_tensor view;
  if (index_add_checks(self, dim, index, source, 1, &d, &view)) return 0;
  return scatter_ws_bytes(self, d, &view, source, deterministic);
}

tx_status tx_index_add_(const tx_tensor* self, int64_t dim, const tx_tensor* index, const tx_tensor* source, double alpha_f,
                        int64_t alpha_i, int alpha_is_int, int deterministic, void* ws, size_t ws_bytes, void* stream) {
  int d;
  tx_tensor view;
  tx_status rc = index_add_checks(self, dim, index, source, alpha_is_int, &d, &view);
  if (rc) return rc;
  set_path("");
  const Alpha alpha{(float)(alpha_is_int ? (double)alpha_i : alpha_f), alpha_is_int ? alpha_i : 0};   // bool: zero or not
  if (index_validation_on() && numel(index) &&
      (rc = validate_index(index, 0, self->ndim ? self->sizes[d] : 1, "index_add_", as_stream(stream)))) return rc;
  return scatter_core("index_add_", self, d, &view, source, alpha, deterministic, ws, ws_bytes, as_stream(stream));
}

}  // extern "C"
