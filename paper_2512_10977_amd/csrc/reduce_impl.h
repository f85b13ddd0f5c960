// Dimension reductions: planner, kernels and launch code.  Included by the
// translation units that instantiate groups of (op, dtype) policies.
//
// A reduction is described as outputs o in [0, nout) x reduced elements r in
// [0, nred); kept dims and reduced dims each stay in logical order (argmax
// needs the logical position) and adjacent dims are merged where strides
// allow.  Two kernels cover every case:
//   rows : a group of G lanes (a wave, or the whole 256-lane workgroup) owns
//          one output and strides through the reduced elements with 16-byte
//          loads when the innermost reduced dim is contiguous; wave-level
//          shuffles, then LDS across waves, combine the lanes.
//   cols : lanes run along the contiguous KEPT dim, each lane owning VEC
//          adjacent outputs and looping over the reduced elements, so every
//          load is coalesced and no cross-lane combine exists.
// When there are too few outputs to fill the chip the reduced range is split
// S ways: pass 1 writes accumulator partials to the workspace, pass 2 (a tiny
// kernel) combines the S partials per output and finalises.
#pragma once
#include <algorithm>
#include <cstring>
#include <type_traits>

#include "common.h"
#include "math_fp.h"

namespace tx {
namespace red {

constexpr int kBlock = 256;
constexpr int kMaxSplit = 1024;

struct Plan {
  int kind;                         // 0 rows, 1 cols
  int nk, nr;                       // merged kept / reduced dims
  int64_t ksize[TX_MAX_DIMS], kxs[TX_MAX_DIMS], kos[TX_MAX_DIMS];
  int64_t rsize[TX_MAX_DIMS], rxs[TX_MAX_DIMS];
  int64_t nout, nred;
  int single_dim;                   // argmax position = coordinate along the one reduced dim (== r)
  int vec;                          // elements per load (1 or 16/sizeof(T))
  int group;                        // rows: lanes per output (32, 64 or 256)
  int nv;                           // cols: vectors per thread (1, 2 or 4)
  double aux;                       // per-op switch handed to Policy::finish (std: 1 = square root; any / all: 1 = all)
  int split;                        // S
  int64_t chunk;                    // reduced elements per split
  int64_t blocks_x;
};

struct Args {
  const char* x;
  char* out;
  char* ws;
  int out_dtype;
  int nk, nr;
  FastDiv kdiv[TX_MAX_DIMS];
  int64_t kxs[TX_MAX_DIMS], kos[TX_MAX_DIMS];
  FastDiv rdiv[TX_MAX_DIMS];
  int64_t rxs[TX_MAX_DIMS];
  int64_t nout, nred, chunk;
  int split, group;
  double correction;
  double aux;                   // see Plan::aux
};

// ---------------------------------------------------------------------------
// accumulator policies.  value_t is what an element is converted to on load.
// ---------------------------------------------------------------------------
template <class T> struct IsFloatT { static constexpr bool value = std::is_same<T, float>::value || std::is_same<T, f16>::value || std::is_same<T, bf16>::value; };

template <class T, bool MEAN> struct SumPolicy {
  using In = T;
  static constexpr bool flt = IsFloatT<T>::value;
  using Acc = typename std::conditional<flt, float, int64_t>::type;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() { return Acc(0); }
  __device__ static void step(Acc& a, T x, int64_t, double) { a += cvt<Acc>(x); }
  __device__ static void merge(Acc& a, const Acc& b) { a += b; }
  __device__ static Acc shfl(const Acc& a, int m) { return shfl_xor(a, m); }
  __device__ static void finish(const Acc& a, int64_t n, double, double, double* f, int64_t* i) {
    if constexpr (flt) *f = MEAN ? (n ? (double)a / (double)n : __longlong_as_double(0x7ff8000000000000ll)) : (double)a;
    else *i = a;
  }
};

template <class T> struct ProdPolicy {
  using In = T;
  static constexpr bool flt = IsFloatT<T>::value;
  using Acc = typename std::conditional<flt, double, int64_t>::type;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() { return Acc(1); }
  __device__ static void step(Acc& a, T x, int64_t, double) {
    if constexpr (flt) a *= cvt<double>(x);
    else a = (int64_t)((uint64_t)a * (uint64_t)cvt<int64_t>(x));
  }
  __device__ static void merge(Acc& a, const Acc& b) {
    if constexpr (flt) a *= b;
    else a = (int64_t)((uint64_t)a * (uint64_t)b);
  }
  __device__ static Acc shfl(const Acc& a, int m) { return shfl_xor(a, m); }
  __device__ static void finish(const Acc& a, int64_t, double, double, double* f, int64_t* i) {
    if constexpr (flt) *f = a; else *i = a;
  }
};

// MIN = true: amin (the same policy with the order reversed)
template <class T, bool MIN = false> struct AmaxPolicy {
  using In = T;
  static constexpr bool flt = IsFloatT<T>::value;
  using Acc = typename std::conditional<flt, float, int64_t>::type;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() {
    if constexpr (flt) return __uint_as_float(MIN ? 0x7f800000u : 0xff800000u);
    else return MIN ? (Acc)0x7fffffffffffffffll : (Acc)0x8000000000000000ll;
  }
  __device__ static bool beats(Acc b, Acc a) { return MIN ? b < a : b > a; }
  __device__ static void merge(Acc& a, const Acc& b) {
    if constexpr (flt) a = (a != a) ? a : ((b != b) ? b : (beats(b, a) ? b : a));
    else a = beats(b, a) ? b : a;
  }
  __device__ static void step(Acc& a, T x, int64_t, double) { merge(a, cvt<Acc>(x)); }
  __device__ static Acc shfl(const Acc& a, int m) { return shfl_xor(a, m); }
  __device__ static void finish(const Acc& a, int64_t, double, double, double* f, int64_t* i) {
    if constexpr (flt) *f = a; else *i = a;
  }
};

template <class V> struct ArgAcc { V v; int64_t i; };
// MIN = true: argmin
template <class T, bool MIN = false> struct ArgmaxPolicy {
  using In = T;
  static constexpr bool flt = IsFloatT<T>::value;
  using V = typename std::conditional<flt, float, int64_t>::type;
  using Acc = ArgAcc<V>;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() {
    Acc a;
    if constexpr (flt) a.v = __uint_as_float(MIN ? 0x7f800000u : 0xff800000u);
    else a.v = MIN ? (V)0x7fffffffffffffffll : (V)0x8000000000000000ll;
    a.i = 0x7fffffffffffffffll;
    return a;
  }
  __device__ static bool beats(V v1, V v2) { return MIN ? v1 < v2 : v1 > v2; }
  // does (v1,i1) outrank (v2,i2)?  NaN outranks everything; ties go to the lower index
  __device__ static bool better(V v1, int64_t i1, V v2, int64_t i2) {
    if constexpr (flt) {
      bool n1 = v1 != v1, n2 = v2 != v2;
      if (n1 || n2) return (n1 && n2) ? i1 < i2 : n1;
    }
    return beats(v1, v2) || (v1 == v2 && i1 < i2);
  }
  __device__ static void merge(Acc& a, const Acc& b) { if (better(b.v, b.i, a.v, a.i)) a = b; }
  // a lane meets its elements in increasing position, so within a lane a strict comparison keeps the
  // earliest of equal values (and the first NaN) without looking at the index
  __device__ static void step(Acc& a, T x, int64_t pos, double) {
    V v = cvt<V>(x);
    bool take;
    if constexpr (flt) take = !(a.v != a.v) && (beats(v, a.v) || v != v);
    else take = beats(v, a.v);
    if (take) { a.v = v; a.i = pos; }
  }
  __device__ static Acc shfl(const Acc& a, int m) { Acc r; r.v = shfl_xor(a.v, m); r.i = shfl_xor(a.i, m); return r; }
  // an untouched index means nothing beat the initial extreme value: every element equals it, the first one wins
  __device__ static void finish(const Acc& a, int64_t, double, double, double*, int64_t* i) {
    *i = a.i == 0x7fffffffffffffffll ? 0 : a.i;
  }
};

// any / all: two bits per accumulator (some element non-zero, every element non-zero); finish picks one.
// NaN counts as non-zero.
struct AnyAllAcc { uint32_t any, all; };
template <class T> struct AnyAllPolicy {
  using In = T;
  static constexpr bool flt = false;                 // integer-style store (bool out)
  using Acc = AnyAllAcc;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() { return Acc{0u, 1u}; }
  __device__ static void step(Acc& a, T x, int64_t, double) {
    uint32_t t;
    if constexpr (IsFloatT<T>::value) t = cvt<float>(x) != 0.0f;
    else t = x != 0;
    a.any |= t;
    a.all &= t;
  }
  __device__ static void merge(Acc& a, const Acc& b) { a.any |= b.any; a.all &= b.all; }
  __device__ static Acc shfl(const Acc& a, int m) { return Acc{shfl_xor(a.any, m), shfl_xor(a.all, m)}; }
  __device__ static void finish(const Acc& a, int64_t, double, double want_all, double*, int64_t* i) {
    *i = want_all != 0.0 ? a.all : a.any;
  }
};

// logsumexp as a running (maximum, sum of exp(x - maximum)) pair; pairs merge by rescaling the smaller side.
// A NaN maximum is sticky; an infinite maximum is the result itself.
struct LseAcc { float m, s; };
template <class T> struct LsePolicy {
  using In = T;
  static constexpr bool flt = true;
  using Acc = LseAcc;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() { return Acc{__uint_as_float(0xff800000u), 0.0f}; }
  // a NaN seen so far lives in s (step) or in m; merge makes both NaN
  __device__ static void merge(Acc& a, const Acc& b) {
    if (a.m != a.m || a.s != a.s || b.m != b.m || b.s != b.s) {
      a.m = a.s = __uint_as_float(0x7fc00000u);
      return;
    }
    const float M = b.m > a.m ? b.m : a.m;
    if (M == __uint_as_float(0xff800000u)) return;             // both empty / all -inf so far
    if (M == __uint_as_float(0x7f800000u)) { a.m = M; a.s = 1.0f; return; }
    a.s = a.s * expf(a.m - M) + b.s * expf(b.m - M);            // exp(-inf) = 0 for a side that is still empty
    a.m = M;
  }
  // one element without branches: e = exp(-|v - m|) (1 when v == m, which covers equal infinities);
  // v <= m: s += e, else s = s e + 1 and m = v.  exp(-inf) = 0 handles the empty state and +inf; a NaN element
  // makes s NaN for good.  Hardware exp2: its relative error (~1e-7 |v - m|) only matters for terms near 1.
  __device__ static void step(Acc& a, T x, int64_t, double) {
    const float v = cvt<float>(x);
    const float d = v == a.m ? 0.0f : -__builtin_fabsf(v - a.m);
    const float e = __expf(d);
    const bool le = v <= a.m;
    a.s = __builtin_fmaf(e, le ? 1.0f : a.s, le ? a.s : 1.0f);
    a.m = __builtin_fmaxf(a.m, v);
  }
  // N consecutive elements at once (the row kernels): the maximum moves first, the old sum is rescaled once, and the
  // N exponentials are independent of each other - a lane's chain is one rescale and N additions per vector instead
  // of N dependent steps.  The differences are taken against the maximum clamped to the finite range, so that an
  // infinite maximum gives exp(+inf) = inf or exp(-inf) = 0 and never inf - inf (finish returns an infinite maximum as it
  // is; only a NaN element makes s NaN).
  template <int N> __device__ static void step_n(Acc& a, const Vec<T, N>& x) {
    float v[N];
    float M = a.m;
#pragma unroll
    for (int e = 0; e < N; ++e) {
      v[e] = cvt<float>(x.v[e]);
      M = __builtin_fmaxf(M, v[e]);
    }
    const float Ms = __builtin_fminf(__builtin_fmaxf(M, -3.4028234663852886e38f), 3.4028234663852886e38f);
    float s = a.s * __expf(a.m - Ms);
#pragma unroll
    for (int e = 0; e < N; ++e) s += __expf(v[e] - Ms);
    a.s = s;
    a.m = M;
  }
  __device__ static Acc shfl(const Acc& a, int m) { return Acc{shfl_xor(a.m, m), shfl_xor(a.s, m)}; }
  __device__ static void finish(const Acc& a, int64_t, double, double, double* f, int64_t*) {
    const bool inf = a.m == __uint_as_float(0x7f800000u) || a.m == __uint_as_float(0xff800000u);
    const bool nan = a.m != a.m || a.s != a.s;
    *f = nan ? (double)__uint_as_float(0x7fc00000u) : inf ? (double)a.m : (double)a.m + (double)logf(a.s);
  }
};

// variance from sums of (x - K) and (x - K)^2 in binary64; K is the first
// element of the reduced range, which keeps the two sums small
struct VarAcc { double s1, s2; };
template <class T> struct VarPolicy {
  using In = T;
  static constexpr bool flt = true;
  using Acc = VarAcc;
  static constexpr bool needs_shift = true;
  __device__ static Acc init() { return Acc{0.0, 0.0}; }
  __device__ static void step(Acc& a, T x, int64_t, double K) {
    double d = cvt<double>(x) - K;
    a.s1 += d;
    a.s2 = __builtin_fma(d, d, a.s2);
  }
  __device__ static void merge(Acc& a, const Acc& b) { a.s1 += b.s1; a.s2 += b.s2; }
  __device__ static Acc shfl(const Acc& a, int m) { return Acc{shfl_xor(a.s1, m), shfl_xor(a.s2, m)}; }
  __device__ static void finish(const Acc& a, int64_t n, double correction, double take_sqrt, double* f, int64_t*) {
    double nn = (double)n;
    double div = nn - correction;
    if (div < 0.0) div = 0.0;
    double m2 = a.s2 - a.s1 * a.s1 / nn;
    if (m2 < 0.0) m2 = 0.0;
    double v = n ? m2 / div : __longlong_as_double(0x7ff8000000000000ll);
    *f = take_sqrt != 0.0 ? __builtin_sqrt(v) : v;           // std
  }
};

// nansum (MEAN = false) / nanmean: the elements that are not NaN, and how many they are
struct NanAcc { float s; int64_t n; };
template <class T, bool MEAN> struct NanSumPolicy {
  using In = T;
  static constexpr bool flt = true;
  using Acc = NanAcc;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() { return Acc{0.0f, 0}; }
  __device__ static void step(Acc& a, T x, int64_t, double) {
    const float v = cvt<float>(x);
    const bool ok = v == v;
    a.s += ok ? v : 0.0f;
    a.n += ok;
  }
  __device__ static void merge(Acc& a, const Acc& b) { a.s += b.s; a.n += b.n; }
  __device__ static Acc shfl(const Acc& a, int m) { return Acc{shfl_xor(a.s, m), shfl_xor(a.n, m)}; }
  __device__ static void finish(const Acc& a, int64_t, double, double, double* f, int64_t*) {
    *f = MEAN ? (double)a.s / (double)a.n : (double)a.s;          // 0 / 0 = NaN: nothing but NaNs, or nothing at all
  }
};

// count_nonzero: a NaN is not zero, -0.0 is
template <class T> struct CountPolicy {
  using In = T;
  static constexpr bool flt = false;                 // int64 out
  using Acc = int64_t;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() { return 0; }
  __device__ static void step(Acc& a, T x, int64_t, double) {
    if constexpr (IsFloatT<T>::value) a += cvt<float>(x) != 0.0f;
    else a += x != 0;
  }
  __device__ static void merge(Acc& a, const Acc& b) { a += b; }
  __device__ static Acc shfl(const Acc& a, int m) { return shfl_xor(a, m); }
  __device__ static void finish(const Acc& a, int64_t, double, double, double*, int64_t* i) { *i = a; }
};

// vector p-norm.  ORD 0: the count of non-zero elements; 1: sum |x| (fp32, like sum); 2: sqrt of the sum of squares
// (binary64, so the squares of large fp32 values do not overflow); 3 / 4: the largest / smallest |x|, NaN if any;
// 5: (sum |x|^p)^(1/p) in binary64 with p arriving as the op's parameter.
template <class T, int ORD> struct NormPolicy {
  using In = T;
  static constexpr bool flt = true;
  using Acc = typename std::conditional<ORD == 0, int64_t, typename std::conditional<ORD == 2 || ORD == 5, double, float>::type>::type;
  static constexpr bool needs_shift = false;
  __device__ static Acc init() {
    if constexpr (ORD == 3) return 0.0f;                               // |x| >= 0
    else if constexpr (ORD == 4) return __uint_as_float(0x7f800000u);
    else return Acc(0);
  }
  __device__ static void merge(Acc& a, const Acc& b) {
    if constexpr (ORD == 3) a = (a != a) ? a : ((b != b) ? b : (b > a ? b : a));
    else if constexpr (ORD == 4) a = (a != a) ? a : ((b != b) ? b : (b < a ? b : a));
    else a += b;
  }
  __device__ static void step(Acc& a, T x, int64_t, double p) {
    const float v = __builtin_fabsf(cvt<float>(x));
    if constexpr (ORD == 0) a += v != 0.0f;
    else if constexpr (ORD == 1) a += v;
    else if constexpr (ORD == 2) a = __builtin_fma((double)v, (double)v, a);
    else if constexpr (ORD == 5) a += pow_abs_d((double)v, p);
    else merge(a, v);
  }
  __device__ static Acc shfl(const Acc& a, int m) { return shfl_xor(a, m); }
  __device__ static void finish(const Acc& a, int64_t, double p, double, double* f, int64_t*) {
    if constexpr (ORD == 2) *f = __builtin_sqrt(a);
    else if constexpr (ORD == 5) *f = pow(a, 1.0 / p);
    else *f = (double)a;
  }
};

// store a finished value in the run-time output dtype
template <bool FLT> __device__ __forceinline__ void store_result(char* out, int64_t off, int dt, double f, int64_t i) {
  if constexpr (FLT) {
    switch (dt) {
      case TX_F32: ((float*)out)[off] = (float)f; break;
      case TX_BF16: ((bf16*)out)[off] = float_to_bf16((float)f); break;
      case TX_F16: ((f16*)out)[off] = (f16)(float)f; break;
      default: ((int64_t*)out)[off] = i; break;
    }
  } else {
    switch (dt) {
      case TX_I64: ((int64_t*)out)[off] = i; break;
      case TX_I32: ((int32_t*)out)[off] = (int32_t)i; break;
      default: ((uint8_t*)out)[off] = (uint8_t)(i != 0); break;
    }
  }
}

template <class P> __device__ __forceinline__ void emit(const Args& a, const typename P::Acc& acc, int64_t oo) {
  double f = 0.0;
  int64_t i = 0;
  P::finish(acc, a.nred, a.correction, a.aux, &f, &i);
  // argmax produces an index even for float input
  if constexpr (std::is_same<typename P::Acc, ArgAcc<float>>::value || std::is_same<typename P::Acc, ArgAcc<int64_t>>::value)
    ((int64_t*)a.out)[oo] = i;
  else
    store_result<P::flt>(a.out, oo, a.out_dtype, f, i);
}

__device__ __forceinline__ int64_t reduced_offset(const Args& a, int64_t r) {
  if (a.nr == 1) return r * a.rxs[0];
  int64_t off = 0;
  uint32_t rem = (uint32_t)r;
  for (int d = a.nr - 1; d >= 0; --d) {
    uint32_t q, m;
    a.rdiv[d].divmod(rem, q, m);
    rem = q;
    off += (int64_t)m * a.rxs[d];
  }
  return off;
}
// Offset of reduced index r, specialised at compile time for the common case of one merged reduced dim
// (the general form walks a table in kernel-argument memory, a dependent scalar load per dim, and that
// between every two vector loads).
template <bool ONE_DIM> struct ReducedOffset {
  const Args& a;
  int64_t s0;
  __device__ __forceinline__ explicit ReducedOffset(const Args& args) : a(args), s0(args.rxs[0]) {}
  __device__ __forceinline__ int64_t operator()(int64_t r) const {
    if constexpr (ONE_DIM) return r * s0;
    else return reduced_offset(a, r);
  }
};

__device__ __forceinline__ void kept_offsets(const Args& a, int64_t o, int64_t* xo, int64_t* oo) {
  int64_t x = 0, y = 0;
  if (a.nk == 1) { x = o * a.kxs[0]; y = o * a.kos[0]; }
  else {
    uint32_t rem = (uint32_t)o;
    for (int d = a.nk - 1; d >= 0; --d) {
      uint32_t q, m;
      a.kdiv[d].divmod(rem, q, m);
      rem = q;
      x += (int64_t)m * a.kxs[d];
      y += (int64_t)m * a.kos[d];
    }
  }
  *xo = x;
  *oo = y;
}

// one vector of a row: a policy may take the whole vector in one call (step_n), else its elements go one by one
template <class P, int N, class = void> struct HasStepN : std::false_type {};
template <class P, int N> struct HasStepN<P, N, std::void_t<decltype(&P::template step_n<N>)>> : std::true_type {};
template <class P, class T, int VEC>
__device__ __forceinline__ void step_vec(typename P::Acc& acc, const Vec<T, VEC>& v, int64_t pos, double K) {
  if constexpr (HasStepN<P, VEC>::value) {
    P::template step_n<VEC>(acc, v);
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e) P::step(acc, v.v[e], pos + e, K);
  }
}

// ---------------------------------------------------------------------------
// rows kernel: grid.x = ceil(nout / groups_per_block), grid.y = split
// ---------------------------------------------------------------------------
template <class P, int VEC, bool ONE_DIM>
__global__ __launch_bounds__(kBlock) void reduce_rows_kernel(const Args a) {
  using T = typename P::In;
  using Acc = typename P::Acc;
  __shared__ Acc lds[kBlock / kWave];
  const int G = a.group;
  const int gpb = kBlock / G;                          // outputs per workgroup
  const int gidx = threadIdx.x / G, lane = threadIdx.x % G;
  const int64_t o = (int64_t)blockIdx.x * gpb + gidx;
  const bool live = o < a.nout;
  int64_t xo = 0, oo = 0;
  if (live) kept_offsets(a, o, &xo, &oo);
  const int64_t begin = (int64_t)blockIdx.y * a.chunk;
  int64_t end = begin + a.chunk;
  if (end > a.nred) end = a.nred;
  const T* x = (const T*)a.x + xo;
  const ReducedOffset<ONE_DIM> roff(a);
  double K = a.correction;                             // policies without a shift receive the op's parameter here
  if constexpr (P::needs_shift) {
    K = 0.0;
    if (live && a.nred > 0) K = cvt<double>(x[roff(0)]);
  }
  Acc acc = P::init();
  if (live) {
    // four loads are issued before the first value is used: a loop that loads, waits and accumulates one
    // vector at a time leaves a single load in flight per wave
    constexpr int kUnroll = 4;
    const int64_t stride = (int64_t)G * VEC;
    int64_t r = begin + (int64_t)lane * VEC;
    for (; r + (kUnroll - 1) * stride < end; r += kUnroll * stride) {
      Vec<T, VEC> v[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) v[u] = vec_load<T, VEC, true>(x + roff(r + u * stride));
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) step_vec<P, T, VEC>(acc, v[u], r + u * stride, K);
    }
    if (r + stride < end) {                    // two left (short rows never enter the loop above)
      Vec<T, VEC> v0 = vec_load<T, VEC, true>(x + roff(r)), v1 = vec_load<T, VEC, true>(x + roff(r + stride));
      step_vec<P, T, VEC>(acc, v0, r, K);
      step_vec<P, T, VEC>(acc, v1, r + stride, K);
      r += 2 * stride;
    }
    for (; r < end; r += stride) {
      Vec<T, VEC> v = vec_load<T, VEC, true>(x + roff(r));
      step_vec<P, T, VEC>(acc, v, r, K);
    }
  }
  // lanes of a group (a wave, or half a wave for short rows: the exchange then stays inside each half)
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) {
    if (m < G) { Acc other = P::shfl(acc, m); P::merge(acc, other); }
  }
  if (G == kBlock) {
    const int w = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) lds[w] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      acc = lds[0];
      for (int k = 1; k < kBlock / kWave; ++k) P::merge(acc, lds[k]);
    }
  }
  if (lane == 0 && live) {
    if (a.split == 1) emit<P>(a, acc, oo);
    else ((Acc*)a.ws)[o * a.split + blockIdx.y] = acc;
  }
}

// ---------------------------------------------------------------------------
// cols kernel: lanes along the innermost kept dim; grid.y = split.  A thread owns NV vectors of VEC
// consecutive outputs, the vectors one workgroup-width apart: per reduced index the workgroup reads
// NV x 256 x VEC contiguous elements, and each lane has NV independent loads in flight per step.
// ---------------------------------------------------------------------------
template <class P, int VEC, int NV, bool ONE_DIM>
__global__ __launch_bounds__(kBlock) void reduce_cols_kernel(const Args a) {
  using T = typename P::In;
  using Acc = typename P::Acc;
  const int64_t first = (int64_t)blockIdx.x * (kBlock * NV * VEC) + (int64_t)threadIdx.x * VEC;
  if (first >= a.nout) return;
  // vectors past the end are clamped onto the thread's first one: loaded again, never written
  int64_t xo[NV], oo[NV];
  bool live[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int64_t o0 = first + (int64_t)j * kBlock * VEC;
    live[j] = o0 < a.nout;
    kept_offsets(a, live[j] ? o0 : first, &xo[j], &oo[j]);
  }
  const T* x = (const T*)a.x;
  const ReducedOffset<ONE_DIM> roff(a);
  const int64_t begin = (int64_t)blockIdx.y * a.chunk;
  int64_t end = begin + a.chunk;
  if (end > a.nred) end = a.nred;
  double K[NV][VEC];
  Acc acc[NV][VEC];
#pragma unroll
  for (int j = 0; j < NV; ++j)
#pragma unroll
    for (int e = 0; e < VEC; ++e) { acc[j][e] = P::init(); K[j][e] = P::needs_shift ? 0.0 : a.correction; }
  if constexpr (P::needs_shift) {
    if (a.nred > 0) {
      const int64_t off = roff(0);
#pragma unroll
      for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int e = 0; e < VEC; ++e) K[j][e] = cvt<double>(x[xo[j] + off + e]);
    }
  }
  // Rolling window, 8 vector loads in flight per lane: each step consumes the oldest reduced index and at
  // once issues the load that is kDepth indices ahead.  (Issuing the 8 loads of a window back to back was
  // measured 25 % slower for bf16 on this shape: they sit a power-of-two stride apart and reach the same
  // DRAM banks together; spread over the accumulate steps they do not.)
  constexpr int kDepth = 8 / NV;
  int64_t r = begin;
  if constexpr (NV == 1) {
    // one vector per thread: the plain loop, unrolled by the compiler, measured fastest (82 us against 112 us
    // for the rolling window on amax of bf16 [64,4096,1024] over dim 0)
#pragma unroll 8
    for (; r < end; ++r) {
      Vec<T, VEC> v = vec_load<T, VEC, true>(x + xo[0] + reduced_offset(a, r));
#pragma unroll
      for (int e = 0; e < VEC; ++e) P::step(acc[0][e], v.v[e], r, K[0][e]);
    }
  } else if (end - begin >= kDepth) {
    Vec<T, VEC> v[kDepth][NV];
#pragma unroll
    for (int u = 0; u < kDepth; ++u) {
      const int64_t off = roff(r + u);
#pragma unroll
      for (int j = 0; j < NV; ++j) v[u][j] = vec_load<T, VEC, true>(x + xo[j] + off);
    }
    for (; r + 2 * kDepth <= end; r += kDepth) {
#pragma unroll
      for (int u = 0; u < kDepth; ++u) {
#pragma unroll
        for (int j = 0; j < NV; ++j)
#pragma unroll
          for (int e = 0; e < VEC; ++e) P::step(acc[j][e], v[u][j].v[e], r + u, K[j][e]);
        const int64_t off = roff(r + u + kDepth);
#pragma unroll
        for (int j = 0; j < NV; ++j) v[u][j] = vec_load<T, VEC, true>(x + xo[j] + off);
      }
    }
#pragma unroll
    for (int u = 0; u < kDepth; ++u)
#pragma unroll
      for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int e = 0; e < VEC; ++e) P::step(acc[j][e], v[u][j].v[e], r + u, K[j][e]);
    r += kDepth;
  }
  for (; r < end; ++r) {
    const int64_t off = roff(r);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      Vec<T, VEC> v = vec_load<T, VEC, true>(x + xo[j] + off);
#pragma unroll
      for (int e = 0; e < VEC; ++e) P::step(acc[j][e], v.v[e], r, K[j][e]);
    }
  }
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    if (!live[j]) continue;
    const int64_t o0 = first + (int64_t)j * kBlock * VEC;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      if (a.split == 1) emit<P>(a, acc[j][e], oo[j] + e);     // innermost kept dim has unit output stride when VEC > 1
      else ((Acc*)a.ws)[(o0 + e) * a.split + blockIdx.y] = acc[j][e];
    }
  }
}

// pass 2: one wave per output; lanes stride over its S partials, then a shuffle tree
template <class P>
__global__ __launch_bounds__(kBlock) void reduce_final_kernel(const Args a) {
  using Acc = typename P::Acc;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t o = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  if (o >= a.nout) return;                               // whole waves leave together
  const Acc* p = (const Acc*)a.ws + o * a.split;
  Acc acc = P::init();
  for (int s = lane; s < a.split; s += kWave) P::merge(acc, p[s]);
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) { Acc other = P::shfl(acc, m); P::merge(acc, other); }
  if (lane == 0) {
    int64_t xo, oo;
    kept_offsets(a, o, &xo, &oo);
    emit<P>(a, acc, oo);
  }
}

// ---------------------------------------------------------------------------
// host: planning
// ---------------------------------------------------------------------------
tx_status normalise_dims(int nd, const int64_t* dims, int ndims, bool* reduced);
// Fills the dim lists of `p` from x / out and the reduced-dim mask.
void plan_dims(Plan* p, const tx_tensor* x, const tx_tensor* out, const bool* reduced, int keepdim);
// Chooses kernel kind, vector width, group, split.  esize = sizeof(input element), acc_size = sizeof(Acc).
void plan_launch(Plan* p, const tx_tensor* x, int esize, bool shift_needs_first);
size_t plan_ws_bytes(const Plan& p, size_t acc_size);

template <class P> tx_status launch(const Plan& p, const tx_tensor* x, const tx_tensor* out, double correction, void* ws,
                                    size_t ws_bytes, hipStream_t stream) {
  using T = typename P::In;
  constexpr int V = 16 / sizeof(T);
  Args a;
  a.x = (const char*)x->data;
  a.out = (char*)out->data;
  a.ws = (char*)ws;
  a.out_dtype = out->dtype;
  a.nk = p.nk;
  a.nr = p.nr;
  for (int d = 0; d < p.nk; ++d) { a.kdiv[d] = FastDiv((uint32_t)p.ksize[d]); a.kxs[d] = p.kxs[d]; a.kos[d] = p.kos[d]; }
  for (int d = 0; d < p.nr; ++d) { a.rdiv[d] = FastDiv((uint32_t)p.rsize[d]); a.rxs[d] = p.rxs[d]; }
  a.nout = p.nout;
  a.nred = p.nred;
  a.chunk = p.chunk;
  a.split = p.split;
  a.group = p.group;
  a.correction = correction;
  a.aux = p.aux;
  if (p.split > 1) {
    size_t need = plan_ws_bytes(p, sizeof(typename P::Acc));
    if (!ws || ws_bytes < need) return fail(TX_ERR_WORKSPACE, "reduce needs %zu workspace bytes, got %zu", need, ws_bytes);
  }
  dim3 grid((unsigned)p.blocks_x, (unsigned)p.split);
  const bool one = p.nr == 1;
  if (p.kind == 0) {
    set_path(p.split > 1 ? "rows-split" : (p.group == kBlock ? "rows-block" : p.group < kWave ? "rows-half" : "rows-wave"));
    if (p.vec > 1 && one) hipLaunchKernelGGL((reduce_rows_kernel<P, V, true>), grid, dim3(kBlock), 0, stream, a);
    else if (p.vec > 1) hipLaunchKernelGGL((reduce_rows_kernel<P, V, false>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((reduce_rows_kernel<P, 1, false>), grid, dim3(kBlock), 0, stream, a);
  } else {
    set_path(p.split > 1 ? "cols-split" : "cols");
    if (p.vec > 1 && p.nv == 4 && one) hipLaunchKernelGGL((reduce_cols_kernel<P, V, 4, true>), grid, dim3(kBlock), 0, stream, a);
    else if (p.vec > 1 && p.nv == 2 && one) hipLaunchKernelGGL((reduce_cols_kernel<P, V, 2, true>), grid, dim3(kBlock), 0, stream, a);
    else if (p.vec > 1 && one) hipLaunchKernelGGL((reduce_cols_kernel<P, V, 1, true>), grid, dim3(kBlock), 0, stream, a);
    else if (p.vec > 1) hipLaunchKernelGGL((reduce_cols_kernel<P, V, 1, false>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((reduce_cols_kernel<P, 1, 1, false>), grid, dim3(kBlock), 0, stream, a);
  }
  tx_status rc = check_launch("reduce kernel");
  if (rc) return rc;
  if (p.split > 1) {
    hipLaunchKernelGGL((reduce_final_kernel<P>), dim3((unsigned)((p.nout + kBlock / kWave - 1) / (kBlock / kWave))), dim3(kBlock), 0,
                       stream, a);
    rc = check_launch("reduce finalise kernel");
  }
  return rc;
}

// per-dtype dispatch for one op family; defined in the translation units
tx_status launch_sum(bool mean, const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_var(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_prod(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_amax(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_argmax(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_amin(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_argmin(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_anyall(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_logsumexp(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_nansum(bool mean, const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_count(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
tx_status launch_norm(const Plan&, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb, hipStream_t s);
size_t acc_size(int op, int dtype);

}  // namespace red
}  // namespace tx
