// Inclusive scans along one dim: the kernels and their launcher, shared by the translation units that instantiate
// them (cumsum in rowops.hip, cumprod and logcumsumexp in scanops.hip).  The combining operation is a template
// parameter; everything sits in an unnamed namespace.
#pragma once
#include <algorithm>
#include <cstring>
#include <type_traits>

#include "common.h"
#include "rows.h"

namespace tx {

// logcumsumexp accumulator: log(sum) = m + log(s), m the largest exponent met and s the sum of exp(x - m).
// An element x is (x, 1), or (0, NaN) for a NaN; nothing is (-inf, 0).
struct LsePair { float m, s; };
template <> struct Cvt<LsePair, float> {
  __device__ __forceinline__ static LsePair run(float v) { return v != v ? LsePair{0.0f, v} : LsePair{v, 1.0f}; }
};
template <> struct Cvt<LsePair, bf16> {
  __device__ __forceinline__ static LsePair run(bf16 v) { return Cvt<LsePair, float>::run(bf16_to_float(v)); }
};
template <> struct Cvt<LsePair, f16> {
  __device__ __forceinline__ static LsePair run(f16 v) { return Cvt<LsePair, float>::run((float)v); }
};
template <> struct Cvt<float, LsePair> {
  // s >= 1 unless nothing or only -inf was met (s = 0, m = -inf: -inf + -inf) or a NaN was (s = NaN)
  __device__ __forceinline__ static float run(LsePair a) { return a.m + __logf(a.s); }
};
template <> struct Cvt<bf16, LsePair> {
  __device__ __forceinline__ static bf16 run(LsePair a) { return float_to_bf16(Cvt<float, LsePair>::run(a)); }
};
template <> struct Cvt<f16, LsePair> {
  __device__ __forceinline__ static f16 run(LsePair a) { return (f16)Cvt<float, LsePair>::run(a); }
};

namespace {

// ---------------------------------------------------------------------------
// the monoid of a scan: cumsum adds, cumprod multiplies (integers wrap), logcumsumexp takes log(e^a + e^b)
// ---------------------------------------------------------------------------
struct ScanAdd {
  template <class A> __device__ __forceinline__ static A id() { return A(0); }
  template <class A> __device__ __forceinline__ static A op(A a, A b) { return a + b; }
};
struct ScanMul {
  template <class A> __device__ __forceinline__ static A id() { return A(1); }
  template <class A> __device__ __forceinline__ static A op(A a, A b) {
    if constexpr (std::is_integral<A>::value) return (A)((unsigned long long)a * (unsigned long long)b);
    else return a * b;
  }
};
struct ScanLse {                                 // on LsePair accumulators
  template <class A> __device__ __forceinline__ static A id() { return LsePair{-__builtin_inff(), 0.0f}; }
  // the sum with the smaller exponent is rescaled to the larger one: one exponential (the other side's factor is 1).
  // The exponent difference is taken as 0 when the two are equal, so equal infinities do not produce inf - inf;
  // exp(-inf) = 0 removes a side that has met nothing (or only -inf), and a NaN sum on either side stays (NaN * 0)
  template <class A> __device__ __forceinline__ static A op(A a, A b) {
    const float d = a.m == b.m ? 0.0f : -__builtin_fabsf(a.m - b.m);
    const float e = __expf(d);
    const bool a_big = a.m >= b.m;
    return LsePair{a_big ? a.m : b.m, __builtin_fmaf(a_big ? b.s : a.s, e, a_big ? a.s : b.s)};
  }
};

// ---------------------------------------------------------------------------
// decoupled look-back scan
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

template <> struct TileState<LsePair> {
  static constexpr int words = 4;
  __device__ static void publish(unsigned long long* st, int64_t tile, uint32_t flag, LsePair v) {
    TileState<int64_t>::publish(st, tile, flag, __builtin_bit_cast(int64_t, v));
  }
  __device__ static uint32_t read(unsigned long long* st, int64_t tile, LsePair* v) {
    int64_t bits;
    const uint32_t f = TileState<int64_t>::read(st, tile, &bits);
    *v = __builtin_bit_cast(LsePair, bits);
    return f;
  }
};
// binary64 accumulators (cumprod of floats) travel as their bit pattern
template <> struct TileState<double> {
  static constexpr int words = 4;
  __device__ static void publish(unsigned long long* st, int64_t tile, uint32_t flag, double v) {
    TileState<int64_t>::publish(st, tile, flag, __double_as_longlong(v));
  }
  __device__ static uint32_t read(unsigned long long* st, int64_t tile, double* v) {
    int64_t bits;
    const uint32_t f = TileState<int64_t>::read(st, tile, &bits);
    *v = __longlong_as_double(bits);
    return f;
  }
};

// zeroes the header and every status word, and tags the header (second word) as a look-back workspace so that
// tx_lookback_status can tell what it is reading
__global__ void scan_clear_kernel(unsigned long long* ws, int64_t words) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < words) ws[i] = i == 1 ? kLookbackMagic : 0ull;
}

struct ScanArgs {
  const char* x;
  char* out;
  char* ws;
  int64_t rows, len, xrow, orow;
  int64_t tiles_per_row, total_tiles;
  int spin_limit;                               // polls of one predecessor's status word before the wait gives up
};

template <class OP, class Acc> __device__ __forceinline__ Acc wave_inclusive(Acc v) {
  const int lane = threadIdx.x & (kWave - 1);
  if constexpr (std::is_same<OP, ScanLse>::value) {
    // logcumsumexp: when the exponents of the wave's lanes lie within 64 of each other (and are finite), every lane
    // rescales its sum to the wave's largest exponent once and the scan is a plain running sum - one exponential per
    // lane instead of two per lane and step.  A lane that has met nothing yet (-inf, 0) rescales to 0 and does not
    // count for the spread; a NaN sum passes through the running sum as it passes through the general form.  Anything
    // else (infinite exponents, a wider spread, where the small sums would lose their bits) takes the general form.
    float M = v.m, lo = v.s == 0.0f ? __builtin_inff() : v.m;
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) {
      M = __builtin_fmaxf(M, shfl_xor(M, d));
      lo = __builtin_fminf(lo, shfl_xor(lo, d));
    }
    if (__builtin_fabsf(M) < __builtin_inff() && M - lo <= 64.0f) {          // the same verdict in every lane
      float s = v.s * __expf(v.m - M);
#pragma unroll
      for (int d = 1; d < kWave; d <<= 1) {
        const float o = shfl_up(s, d);
        if (lane >= d) s += o;
      }
      return Acc{M, s};
    }
  }
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    Acc o = shfl_up(v, d);
    if (lane >= d) v = OP::op(o, v);
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
template <class T, class Acc, int VEC, int THREADS, int NV, class OP = ScanAdd>
__device__ __forceinline__ void scan_tile_load(const T* xt, int64_t left, Acc (&dst)[NV][VEC]) {
  if (left >= (int64_t)THREADS * NV * VEC) {
    scan_tile_load_full<T, Acc, VEC, THREADS, NV>(xt, dst);
  } else {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int64_t c = ((int64_t)k * THREADS + threadIdx.x) * VEC;
#pragma unroll
      for (int e = 0; e < VEC; ++e) dst[k][e] = (c + e < left) ? cvt<Acc>(xt[c + e]) : OP::template id<Acc>();
    }
  }
}
template <class O, class Acc, int VEC, int THREADS, int NV, class OP = ScanAdd>
__device__ __forceinline__ void scan_tile_store_full(O* ot, const Acc (&v)[NV][VEC], const Acc (&add)[NV]) {
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    Vec<O, VEC> tv;
#pragma unroll
    for (int e = 0; e < VEC; ++e) tv.v[e] = cvt<O>((Acc)OP::op(add[k], v[k][e]));
    vec_store<O, VEC, true>(ot + ((int64_t)k * THREADS + threadIdx.x) * VEC, tv);
  }
}
template <class O, class Acc, int VEC, int THREADS, int NV, class OP = ScanAdd>
__device__ __forceinline__ void scan_tile_store(O* ot, int64_t left, const Acc (&v)[NV][VEC], const Acc (&add)[NV]) {
  if (left >= (int64_t)THREADS * NV * VEC) {
    scan_tile_store_full<O, Acc, VEC, THREADS, NV, OP>(ot, v, add);
  } else {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int64_t c = ((int64_t)k * THREADS + threadIdx.x) * VEC;
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (c + e < left) ot[c + e] = cvt<O>((Acc)OP::op(add[k], v[k][e]));
    }
  }
}

// THREADS is 256 or 1024.  Every workgroup draws one ticket from a single counter, and same-address atomics
// retire at roughly one per 12 ns on this chip, so a 16 KiB tile (256 lanes) caps the kernel near 2.7 TB/s of
// traffic; 64 KiB tiles (1024 lanes, same registers per lane) keep the ticket off the critical path.  The
// smaller tile is kept for inputs with too few tiles to fill the chip.  (A ticket counter per row instead - workgroup
// b on row b mod rows - measured no better on [4096,65536] fp32 (352 against 358 us) and worse everywhere else: int64
// 731 against 682 us, 8 rows of 16 Mi 251 against 200 us, cumprod 466 against 351 us.)
// (A 1024-lane workgroup is four waves per SIMD: two of them fit a CU only up to 64 vector registers, and the
// logcumsumexp instance came to 65 with its faster wave scan, which left one workgroup per CU and took 805 us instead
// of 625 us; the second launch bound asks the compiler for 8 waves per SIMD where the accumulators are small enough.)
template <class T, class O, class Acc, int VEC, int THREADS, int NV, class OP = ScanAdd>
__global__ __launch_bounds__(THREADS, (THREADS == 1024 && sizeof(Acc) * VEC <= 32) ? 8 : 1) void cumsum_lookback_kernel(const ScanArgs a) {
  const Acc kId = OP::template id<Acc>();
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
  // in one or two of them, which shortens every look-back chain (row-major tickets - a contiguous window of resident
  // tiles, but each waiting on the tile just before it - measured 365 against 355 us on [4096,65536] fp32, 745 against
  // 685 us on int64, 241 against 200 us on 8 rows of 16 Mi)
  const int64_t t = ticket / a.rows, row = ticket - t * a.rows;
  const int64_t slot = row * a.tiles_per_row + t;      // status word of this tile (row-major)
  const T* x = (const T*)a.x + row * a.xrow + t * kTileElems;
  O* out = (O*)a.out + row * a.orow + t * kTileElems;
  const int64_t left = a.len - t * kTileElems;      // valid elements in this tile (may exceed the tile)
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;

  Acc v[NV][VEC];
  scan_tile_load<T, Acc, VEC, THREADS, NV, OP>(x, left, v);
  Acc excl[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
#pragma unroll
    for (int e = 1; e < VEC; ++e) v[k][e] = OP::op(v[k][e - 1], v[k][e]);
    const Acc incl = wave_inclusive<OP>(v[k][VEC - 1]);
    Acc up = shfl_up(incl, 1);
    excl[k] = lane == 0 ? kId : up;
    if (lane == kWave - 1) wave_tot[k * kWaves + w] = incl;     // tile order: sub-tile k, then wave w
  }
  __syncthreads();
  if (w == 0) {
    // exclusive scan of the wave totals, then the tile's exclusive prefix by look-back
    const Acc tot = lane < kTotals ? wave_tot[lane] : kId;
    const Acc incl = wave_inclusive<OP>(tot);
    const Acc up = shfl_up(incl, 1);
    if (lane < kTotals) wave_tot[lane] = lane == 0 ? kId : up;
    const Acc tile_total = shfl_idx(incl, kTotals - 1);
    Acc prefix = kId;
    if (t == 0) {
      if (lane == 0) TileState<Acc>::publish(status, slot, kPrefix, tile_total);
    } else {
      if (lane == 0) TileState<Acc>::publish(status, slot, kAggregate, tile_total);
      int64_t look = t - 1;                    // nearest predecessor not yet folded in (row-local index)
      bool done = false;
      while (!done) {
        const int64_t mine = look - lane;      // lane i inspects predecessor look - i
        Acc val = kId;
        uint32_t flag = kPrefix;               // positions before the row start count as an empty prefix
        if (mine >= 0) {
          flag = kEmpty;
          for (int spins = 0; spins < a.spin_limit; ++spins) {      // a limit of 0 (host-forced, for tests) gives up at once
            flag = TileState<Acc>::read(status, slot - t + mine, &val);
            if (flag != kEmpty) break;
            __builtin_amdgcn_s_sleep(2);
          }
          if (flag == kEmpty) { hdr->error = 1; flag = kPrefix; val = kId; }
        }
        const unsigned long long has_prefix = __ballot(flag == kPrefix);
        const int stop = __ffsll((long long)has_prefix) - 1;      // nearest predecessor holding a full prefix
        Acc contrib = (mine >= 0 && (stop < 0 || lane <= stop)) ? val : kId;
#pragma unroll
        for (int m = kWave / 2; m >= 1; m >>= 1) contrib = OP::op(contrib, shfl_xor(contrib, m));
        prefix = OP::op(contrib, prefix);
        if (stop >= 0) done = true;
        else look -= kWave;
      }
      if (lane == 0) TileState<Acc>::publish(status, slot, kPrefix, OP::op(prefix, tile_total));
    }
    if (lane == 0) tile_prefix = prefix;
  }
  __syncthreads();
  const Acc p = tile_prefix;
  Acc add[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) add[k] = OP::op(OP::op(p, wave_tot[k * kWaves + w]), excl[k]);
  scan_tile_store<O, Acc, VEC, THREADS, NV, OP>(out, left, v, add);
}

// Row-carry scan: one workgroup walks a whole row tile by tile and carries the running total in registers.
// No inter-workgroup traffic at all, so it is the better choice whenever there are enough rows to fill the
// chip.  The next tile's loads are issued before the current tile is scanned; for tiles that lie wholly
// inside the row every load and store is unconditional, so the wait for the prefetched tile can leave the
// previous tile's stores in flight.
template <class T, class O, class Acc, int VEC, class OP = ScanAdd>
__global__ __launch_bounds__(kBlock) void cumsum_carry_kernel(const ScanArgs a) {
  const Acc kId = OP::template id<Acc>();
  constexpr int kTileElems = kBlock * kNV * VEC;
  constexpr int kWaves = kBlock / kWave;
  __shared__ Acc wave_tot[2][kNV][kWaves];
  const int64_t row = blockIdx.x;
  const T* x = (const T*)a.x + row * a.xrow;
  O* out = (O*)a.out + row * a.orow;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  Acc carry = kId;
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
      scan_tile_load<T, Acc, VEC, kBlock, kNV, OP>(x + (t + 1) * kTileElems, a.len - (t + 1) * kTileElems, nxt);
    const int buf = (int)(t & 1);
    Acc excl[kNV];
#pragma unroll
    for (int k = 0; k < kNV; ++k) {
#pragma unroll
      for (int e = 1; e < VEC; ++e) v[k][e] = OP::op(v[k][e - 1], v[k][e]);
      const Acc incl = wave_inclusive<OP>(v[k][VEC - 1]);
      Acc up = shfl_up(incl, 1);
      excl[k] = lane == 0 ? kId : up;
      if (lane == kWave - 1) wave_tot[buf][k][w] = incl;
    }
    __syncthreads();                       // one barrier per tile: the two LDS buffers alternate
    Acc running = carry;
    Acc add[kNV];
#pragma unroll
    for (int k = 0; k < kNV; ++k) {
#pragma unroll
      for (int ww = 0; ww < kWaves; ++ww) {
        if (ww == w) add[k] = OP::op(running, excl[k]);
        running = OP::op(running, wave_tot[buf][k][ww]);
      }
    }
    carry = running;
    if constexpr (decltype(steady)::value) scan_tile_store_full<O, Acc, VEC, kBlock, kNV, OP>(out + t * kTileElems, v, add);
    else scan_tile_store<O, Acc, VEC, kBlock, kNV, OP>(out + t * kTileElems, a.len - t * kTileElems, v, add);
  };

  scan_tile_load<T, Acc, VEC, kBlock, kNV, OP>(x, a.len, nxt);
  // The first tile must have landed before the steady loop is entered: otherwise the loop's own wait has to
  // cover "loads still pending, nothing issued after them" as well and becomes a full drain, which would also
  // sit out the previous tile's stores on every iteration.  (vmcnt = 0; the other counters are left alone.)
  __builtin_amdgcn_s_waitcnt(0x0F70);
  const int64_t nfull = a.len / kTileElems;          // tiles wholly inside the row: the branch-free path
  int64_t t = 0;
  for (; t + 1 < nfull; ++t) tile(t, std::true_type{});
  for (; t < a.tiles_per_row; ++t) tile(t, std::false_type{});
}

template <class T, class O, class Acc, class OP = ScanAdd>
__global__ __launch_bounds__(kBlock) void cumsum_strided_kernel(const StridedArgs a) {
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (idx >= a.sl.count) return;
  int64_t xo, oo;
  slice_offsets(a.sl, idx, &xo, &oo);
  const T* x = (const T*)a.x + xo;
  O* out = (O*)a.out + oo;
  Acc acc = OP::template id<Acc>();
  for (int64_t j = 0; j < a.len; ++j) {
    acc = OP::op(acc, cvt<Acc>(x[j * a.xs]));
    out[j * a.os] = cvt<O>(acc);
  }
}

struct ScanPlan {
  bool lookback;
  int vec;
  int64_t rows, len, xrow, orow, tiles_per_row, total_tiles;
  size_t ws_bytes;
};

// elements per vector: 16 bytes of input, but at most 8 elements (a bool input with its 8-byte accumulators would
// otherwise hold 64 accumulators per lane and spill them)
template <class T> constexpr int scan_vec() { return sizeof(T) == 1 ? 8 : 16 / (int)sizeof(T); }

template <class T, class O, class Acc> ScanPlan scan_plan(const tx_tensor* out, const tx_tensor* x, int dim, const Slices& sl) {
  constexpr int V = scan_vec<T>();
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

// OP = ScanAdd may hand a scan along a non-innermost dim to the column kernels; the other monoids keep the strided form
template <class T, class O, class Acc, class OP = ScanAdd>
tx_status cumsum_launch(const tx_tensor* out, const tx_tensor* x, int dim, void* ws, size_t ws_bytes, hipStream_t stream,
                        size_t* query) {
  constexpr int V = scan_vec<T>();
  Slices sl;
  build_slices(&sl, x, out, x->ndim ? dim : -1);
  ScanPlan p = scan_plan<T, O, Acc>(out, x, dim, sl);
  if constexpr (std::is_same<OP, ScanAdd>::value)
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
        hipLaunchKernelGGL((cumsum_carry_kernel<T, O, Acc, V, OP>), dim3((unsigned)p.rows), dim3(kBlock), 0, stream, a);
      else
        hipLaunchKernelGGL((cumsum_carry_kernel<T, O, Acc, 1, OP>), dim3((unsigned)p.rows), dim3(kBlock), 0, stream, a);
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
    a.spin_limit = strcmp(forced_path(), "scan-lookback-giveup") ? kSpinLimit : 0;
    const int64_t words = (int64_t)((256 + (size_t)a.total_tiles * TileState<Acc>::words * 8) / 8);   // <= p.ws_bytes / 8
    hipLaunchKernelGGL(scan_clear_kernel, dim3((unsigned)((words + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream,
                       (unsigned long long*)ws, words);
    set_path(p.vec > 1 ? (big ? "scan-lookback-wide" : "scan-lookback") : (big ? "scan-lookback-wide-scalar" : "scan-lookback-scalar"));
    const dim3 grid((unsigned)a.total_tiles);
    if (p.vec > 1 && big)
      hipLaunchKernelGGL((cumsum_lookback_kernel<T, O, Acc, V, kBig, kBigNV, OP>), grid, dim3(kBig), 0, stream, a);
    else if (p.vec > 1)
      hipLaunchKernelGGL((cumsum_lookback_kernel<T, O, Acc, V, kBlock, kNV, OP>), grid, dim3(kBlock), 0, stream, a);
    else if (big)
      hipLaunchKernelGGL((cumsum_lookback_kernel<T, O, Acc, 1, kBig, kBigNV, OP>), grid, dim3(kBig), 0, stream, a);
    else
      hipLaunchKernelGGL((cumsum_lookback_kernel<T, O, Acc, 1, kBlock, kNV, OP>), grid, dim3(kBlock), 0, stream, a);
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
  hipLaunchKernelGGL((cumsum_strided_kernel<T, O, Acc, OP>), dim3((unsigned)((sl.count + kBlock - 1) / kBlock)), dim3(kBlock),
                     0, stream, a);
  return check_launch("cumsum strided kernel");
}

}  // namespace
}  // namespace tx
