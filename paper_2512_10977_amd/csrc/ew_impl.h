// Elementwise machinery shared by the elementwise translation units: typed and
// run-time-typed element access, the functor plumbing, and the operand
// iterator's three kernel paths with their launcher.
//
//   vec     : output inner dim contiguous, every input inner stride 0 or 1.  A
//             workgroup owns one tile of one inner row; lanes move 16-byte
//             vectors; outer offsets are computed once per workgroup in SALU.
//   tile    : 2-D problems where some input runs contiguously along the
//             output's OUTER dim (a transposed view).  64x64 tiles are staged
//             through LDS so both the global reads and writes are coalesced.
//   generic : one element per lane-slot, offsets from a full index
//             decomposition with magic-number division.
//
// Everything here sits in an unnamed namespace: each translation unit
// instantiates the kernels for its own functors.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstring>
#include <type_traits>

#include "common.h"
#include "iter.h"
#include "math_fp.h"

namespace tx {

// second translation unit (elementwise_b.hip)
tx_status ew_pow(const Iter& it, int da, int db, int common, hipStream_t s);
// comparison / logical family written into a non-bool out tensor
tx_status ew_compare_cast(const Iter& it, int code, int common, hipStream_t s);
// unary op whose out dtype differs from the result dtype rd, and logical_not
tx_status ew_unary_cast(const Iter& it, int op, int in_dtype, int rd, hipStream_t s);

// third translation unit (elementwise_c.hip): unary operators from TX_SIN on, bitwise binary operators and atan2
tx_status ew_unary_third(const Iter& it, int op, int in_dtype, int rd, hipStream_t s);
tx_status ew_binary_third(const Iter& it, int op, int da, int db, int common, hipStream_t s);

// fourth translation unit (elementwise_d.hip): unary operators from TX_TAN on, binary operators from TX_FMOD on
tx_status ew_unary_fourth(const Iter& it, int op, int in_dtype, int rd, hipStream_t s);
tx_status ew_binary_fourth(const Iter& it, int op, int da, int db, int common, hipStream_t s);

namespace {

constexpr int kBlock = 256;

// Marker for an operand whose storage dtype is only known at run time and that
// the kernel converts to the compute type CT on load (or from CT on store).
template <class CT> struct Dyn {};

template <class T> struct Elem {
  using value_t = T;
  static constexpr bool dynamic = false;
  static constexpr int static_size = sizeof(T);
  __device__ __forceinline__ static T load(const char* base, int64_t idx, int) { return ((const T*)base)[idx]; }
  template <int E, bool NT> __device__ __forceinline__ static void load_vec(const char* base, int64_t idx, int, T (&out)[E]) {
    Vec<T, E> v = vec_load<T, E, NT>((const T*)base + idx);
#pragma unroll
    for (int e = 0; e < E; ++e) out[e] = v.v[e];
  }
  __device__ __forceinline__ static void store(char* base, int64_t idx, int, T v) { ((T*)base)[idx] = v; }
  template <int E> __device__ __forceinline__ static void store_vec(char* base, int64_t idx, int, const T (&in)[E]) {
    Vec<T, E> v;
#pragma unroll
    for (int e = 0; e < E; ++e) v.v[e] = in[e];
    vec_store<T, E, true>((T*)base + idx, v);
  }
};

template <class S, class CT, int E, bool NT>
__device__ __forceinline__ void load_cvt_vec(const char* base, int64_t idx, CT (&out)[E]) {
  Vec<S, E> v = vec_load<S, E, NT>((const S*)base + idx);
#pragma unroll
  for (int e = 0; e < E; ++e) out[e] = cvt<CT>(v.v[e]);
}
template <class S, class CT, int E>
__device__ __forceinline__ void store_cvt_vec(char* base, int64_t idx, const CT (&in)[E]) {
  Vec<S, E> v;
#pragma unroll
  for (int e = 0; e < E; ++e) v.v[e] = cvt<S>(in[e]);
  vec_store<S, E, true>((S*)base + idx, v);
}

template <> struct Elem<Dyn<float>> {
  using value_t = float;
  static constexpr bool dynamic = true;
  static constexpr int static_size = 0;
  __device__ __forceinline__ static float load(const char* b, int64_t i, int dt) {
    switch (dt) {
      case TX_F32: return ((const float*)b)[i];
      case TX_BF16: return bf16_to_float(((const bf16*)b)[i]);
      case TX_F16: return (float)((const f16*)b)[i];
      case TX_I64: return (float)((const int64_t*)b)[i];
      case TX_I32: return (float)((const int32_t*)b)[i];
      default: return (float)((const uint8_t*)b)[i];
    }
  }
  template <int E, bool NT> __device__ __forceinline__ static void load_vec(const char* b, int64_t i, int dt, float (&o)[E]) {
    switch (dt) {
      case TX_F32: load_cvt_vec<float, float, E, NT>(b, i, o); break;
      case TX_BF16: load_cvt_vec<bf16, float, E, NT>(b, i, o); break;
      case TX_F16: load_cvt_vec<f16, float, E, NT>(b, i, o); break;
      case TX_I64: load_cvt_vec<int64_t, float, E, NT>(b, i, o); break;
      case TX_I32: load_cvt_vec<int32_t, float, E, NT>(b, i, o); break;
      default: load_cvt_vec<uint8_t, float, E, NT>(b, i, o); break;
    }
  }
  __device__ __forceinline__ static void store(char* b, int64_t i, int dt, float v) {
    switch (dt) {
      case TX_F32: ((float*)b)[i] = v; break;
      case TX_BF16: ((bf16*)b)[i] = float_to_bf16(v); break;
      default: ((f16*)b)[i] = (f16)v; break;
    }
  }
  template <int E> __device__ __forceinline__ static void store_vec(char* b, int64_t i, int dt, const float (&in)[E]) {
    switch (dt) {
      case TX_F32: store_cvt_vec<float, float, E>(b, i, in); break;
      case TX_BF16: store_cvt_vec<bf16, float, E>(b, i, in); break;
      default: store_cvt_vec<f16, float, E>(b, i, in); break;
    }
  }
};

template <> struct Elem<Dyn<int64_t>> {
  using value_t = int64_t;
  static constexpr bool dynamic = true;
  static constexpr int static_size = 0;
  __device__ __forceinline__ static int64_t load(const char* b, int64_t i, int dt) {
    switch (dt) {
      case TX_I64: return ((const int64_t*)b)[i];
      case TX_I32: return ((const int32_t*)b)[i];
      default: return ((const uint8_t*)b)[i];
    }
  }
  template <int E, bool NT> __device__ __forceinline__ static void load_vec(const char* b, int64_t i, int dt, int64_t (&o)[E]) {
    switch (dt) {
      case TX_I64: load_cvt_vec<int64_t, int64_t, E, NT>(b, i, o); break;
      case TX_I32: load_cvt_vec<int32_t, int64_t, E, NT>(b, i, o); break;
      default: load_cvt_vec<uint8_t, int64_t, E, NT>(b, i, o); break;
    }
  }
  // an integer / bool result written to any dtype it may be cast to: integers narrow by wrapping and reach the
  // floating dtypes through fp32; TX_BOOL is only ever the target of a 0 / 1 value
  __device__ __forceinline__ static void store(char* b, int64_t i, int dt, int64_t v) {
    switch (dt) {
      case TX_I64: ((int64_t*)b)[i] = v; break;
      case TX_I32: ((int32_t*)b)[i] = (int32_t)v; break;
      case TX_F32: ((float*)b)[i] = (float)v; break;
      case TX_BF16: ((bf16*)b)[i] = float_to_bf16((float)v); break;
      case TX_F16: ((f16*)b)[i] = (f16)(float)v; break;
      default: ((uint8_t*)b)[i] = (uint8_t)v; break;
    }
  }
  template <int E> __device__ __forceinline__ static void store_vec(char* b, int64_t i, int dt, const int64_t (&in)[E]) {
    switch (dt) {
      case TX_I64: store_cvt_vec<int64_t, int64_t, E>(b, i, in); break;
      case TX_I32: store_cvt_vec<int32_t, int64_t, E>(b, i, in); break;
      case TX_BOOL: store_cvt_vec<uint8_t, int64_t, E>(b, i, in); break;
      default: {
        float f[E];
#pragma unroll
        for (int e = 0; e < E; ++e) f[e] = (float)in[e];
        Elem<Dyn<float>>::store_vec<E>(b, i, dt, f);
      }
    }
  }
};

// ---------------------------------------------------------------------------
// functor plumbing: every functor declares Out, In0, In1, In2 (unused inputs
// are `void`) and NIN, and is called with the converted input values.
// ---------------------------------------------------------------------------
template <class T> struct ValueOf { using type = typename Elem<T>::value_t; };
template <> struct ValueOf<void> { using type = uint8_t; };
template <class T> constexpr int static_size_of() {
  if constexpr (std::is_void<T>::value) return 0;
  else return Elem<T>::static_size;
}
template <class T> constexpr bool is_dynamic() {
  if constexpr (std::is_void<T>::value) return false;
  else return Elem<T>::dynamic;
}

template <class F> constexpr int vec_per_lane(decltype(F::VPL)*) { return F::VPL; }
template <class F> constexpr int vec_per_lane(...) { return 1; }

template <class F> struct Shape {
  static constexpr bool dynamic = is_dynamic<typename F::Out>() || is_dynamic<typename F::In0>() ||
                                  is_dynamic<typename F::In1>() || is_dynamic<typename F::In2>();
  static constexpr int s0 = static_size_of<typename F::Out>(), s1 = static_size_of<typename F::In0>(),
                       s2 = static_size_of<typename F::In1>(), s3 = static_size_of<typename F::In2>();
  static constexpr int cmin(int a, int b) { return b == 0 ? a : (a < b ? a : b); }
  static constexpr int cmax(int a, int b) { return a > b ? a : b; }
  static constexpr int min_size = cmin(cmin(cmin(s0 ? s0 : 16, s1), s2), s3);
  static constexpr int max_size = cmax(cmax(cmax(s0, s1), s2), s3);
  // elements per lane per vector: the WIDEST operand moves 16 bytes, so every access of a wave is one
  // contiguous run (narrower operands move 2-8 bytes per lane, still fully coalesced).  Letting the
  // narrowest operand set the width made the wide operands 64-byte-strided per instruction, which halves
  // the throughput of streaming loads.
  static constexpr int E = dynamic ? 4 : (max_size >= 16 ? 1 : 16 / max_size);
  // vectors per lane: one.  On this chip a streaming kernel is fastest with many small waves (a plain copy
  // moves 6.5 TB/s with one 16-byte vector per lane and 5.8 TB/s with four)
  // A functor with enough arithmetic per element to show beside the memory time (a transcendental) may ask for more,
  // by declaring VPL: its workgroup then has the next vector's load in flight while it computes the first.
  static constexpr int per_vec = E * max_size;
  static constexpr int U = vec_per_lane<F>(0);
};

template <class T> struct TypeTag { using type = T; };

// A unary functor may evaluate the E elements of a vector in one call (apply_n): what its formula keeps in vector
// registers - the leading coefficient of a polynomial, which the instruction set cannot take from a scalar register
// beside a second constant - is then set up once per vector and not once per element.
template <class F, int E, class = void> struct HasApplyN : std::false_type {};
template <class F, int E> struct HasApplyN<F, E, std::void_t<decltype(&F::template apply_n<E>)>> : std::true_type {};

template <class F, class A, class B, class C>
__device__ __forceinline__ typename ValueOf<typename F::Out>::type apply(const F& f, A a, B b, C c) {
  if constexpr (F::NIN == 1) return f(a);
  else if constexpr (F::NIN == 2) return f(a, b);
  else return f(a, b, c);
}

// ---------------------------------------------------------------------------
// vec path
// ---------------------------------------------------------------------------
template <int NOPS> struct VecArgs {
  char* data[NOPS];
  int dtype[NOPS];
  int inner_stride[NOPS];                    // 0 or 1 (operand 0 = out: always 1)
  int stream[NOPS];                          // operand is read exactly once (no broadcast dim): non-temporal loads
  int nouter;
  FastDiv tiles_per_row;
  FastDiv osize[TX_MAX_DIMS - 1];            // outer sizes, outer -> inner
  int64_t ostride[NOPS][TX_MAX_DIMS - 1];    // elements
  int64_t n0;                                // inner extent
};

// STREAM is a compile-time flag on purpose: a load whose non-temporal hint depends on a run-time value is
// compiled as a plain load (the two sides of the branch are merged and the hint is dropped).
template <class In, int E, bool STREAM, int NOPS>
__device__ __forceinline__ void vec_fetch(const VecArgs<NOPS>& a, int o, int64_t base, int64_t i, int valid,
                                          typename ValueOf<In>::type (&x)[E]) {
  if constexpr (!std::is_void<In>::value) {
    using EL = Elem<In>;
    if (a.inner_stride[o] == 0) {
      typename EL::value_t v = EL::load(a.data[o], base, a.dtype[o]);
#pragma unroll
      for (int e = 0; e < E; ++e) x[e] = v;
    } else if (valid == E) {
      EL::template load_vec<E, STREAM>(a.data[o], base + i, a.dtype[o], x);
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e)
        if (e < valid) x[e] = EL::load(a.data[o], base + i + e, a.dtype[o]);
    }
  }
}

// The same fetch for a tile that lies wholly inside the row, in two steps so that the loads of all operands are in
// flight together: vec_issue starts the load (an operand with inner stride 0 loads its one element into x[0]),
// vec_spread copies that element to the other slots.  Done in one step, the copies make the wave wait for the
// stride-0 load before the next operand's load is even issued: two memory round trips in a row for a[r] + b[c].
template <class In, int E, bool STREAM, int NOPS>
__device__ __forceinline__ void vec_issue(const VecArgs<NOPS>& a, int o, int64_t base, int64_t i,
                                          typename ValueOf<In>::type (&x)[E]) {
  if constexpr (!std::is_void<In>::value) {
    using EL = Elem<In>;
    if (a.inner_stride[o] == 0) x[0] = EL::load(a.data[o], base, a.dtype[o]);
    else EL::template load_vec<E, STREAM>(a.data[o], base + i, a.dtype[o], x);
  }
}
template <class In, int E, int NOPS>
__device__ __forceinline__ void vec_spread(const VecArgs<NOPS>& a, int o, typename ValueOf<In>::type (&x)[E]) {
  if constexpr (!std::is_void<In>::value) {
    if (a.inner_stride[o] == 0) {
#pragma unroll
      for (int e = 1; e < E; ++e) x[e] = x[0];
    }
  }
}

// STREAM: every input that is read along the inner dim is read exactly once (no broadcast dim anywhere), so
// its loads are marked non-temporal.
template <class F, int E, int U, bool STREAM>
__global__ __launch_bounds__(kBlock) void ew_vec_kernel(const F f, const VecArgs<F::NIN + 1> a) {
  constexpr int NOPS = F::NIN + 1;
  // Everything up to the first vector load is scalar work on kernel arguments.  It is written so that the argument
  // reads have fixed offsets and no read waits for a branch on an earlier one (a chain of dependent scalar loads is a
  // few hundred nanoseconds in which the workgroup has no memory request in flight, and a workgroup only moves a few
  // KiB): up to two outer dims are decomposed by unrolled code (the host pads the unused ones with size 1, stride 0),
  // more by the loop.
  // Naming every argument the common path needs as the input of one empty asm statement makes the compiler fetch them
  // together, ahead of the first branch (it would otherwise fetch each where it is first used, one round trip each).
  asm volatile("" ::"s"(a.tiles_per_row.m), "s"(a.tiles_per_row.s), "s"(a.tiles_per_row.d), "s"(a.nouter), "s"(a.n0),
               "s"(a.osize[0].m), "s"(a.osize[0].s), "s"(a.osize[0].d), "s"(a.osize[1].m), "s"(a.osize[1].s),
               "s"(a.osize[1].d), "s"(a.data[0]), "s"(a.data[1]), "s"(a.ostride[0][0]), "s"(a.ostride[0][1]),
               "s"(a.ostride[1][0]), "s"(a.ostride[1][1]), "s"(a.inner_stride[1]));
  if constexpr (NOPS >= 3)
    asm volatile("" ::"s"(a.data[2]), "s"(a.ostride[2][0]), "s"(a.ostride[2][1]), "s"(a.inner_stride[2]));
  if constexpr (NOPS >= 4)
    asm volatile("" ::"s"(a.data[3]), "s"(a.ostride[3][0]), "s"(a.ostride[3][1]), "s"(a.inner_stride[3]));
  uint32_t outer, tile;
  a.tiles_per_row.divmod(blockIdx.x, outer, tile);
  int64_t base[NOPS];
#pragma unroll
  for (int o = 0; o < NOPS; ++o) base[o] = 0;
  if (a.nouter <= 2) {
#pragma unroll
    for (int d = 1; d >= 0; --d) {
      uint32_t q, r;
      a.osize[d].divmod(outer, q, r);
      outer = q;
#pragma unroll
      for (int o = 0; o < NOPS; ++o) base[o] += (int64_t)r * a.ostride[o][d];
    }
  } else {
    for (int d = a.nouter - 1; d >= 0; --d) {
      uint32_t q, r;
      a.osize[d].divmod(outer, q, r);
      outer = q;
#pragma unroll
      for (int o = 0; o < NOPS; ++o) base[o] += (int64_t)r * a.ostride[o][d];
    }
  }
  const int64_t t0 = (int64_t)tile * (kBlock * E * U);
  const int64_t i0 = t0 + (int64_t)threadIdx.x * E;
  typename ValueOf<typename F::In0>::type x0[U][E];
  typename ValueOf<typename F::In1>::type x1[U][E];
  typename ValueOf<typename F::In2>::type x2[U][E];
  using EO = Elem<typename F::Out>;
  if (t0 + kBlock * E * U <= a.n0) {                      // the whole tile lies inside the row (wave-uniform): no masks
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = i0 + (int64_t)u * kBlock * E;
      vec_issue<typename F::In0, E, STREAM>(a, 1, base[1], i, x0[u]);
      if constexpr (F::NIN >= 2) vec_issue<typename F::In1, E, STREAM>(a, 2, base[2], i, x1[u]);
      if constexpr (F::NIN >= 3) vec_issue<typename F::In2, E, STREAM>(a, 3, base[3], i, x2[u]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      vec_spread<typename F::In0, E>(a, 1, x0[u]);
      if constexpr (F::NIN >= 2) vec_spread<typename F::In1, E>(a, 2, x1[u]);
      if constexpr (F::NIN >= 3) vec_spread<typename F::In2, E>(a, 3, x2[u]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = i0 + (int64_t)u * kBlock * E;
      typename EO::value_t y[E];
      if constexpr (HasApplyN<F, E>::value) {
        f.template apply_n<E>(x0[u], y);
      } else {
#pragma unroll
        for (int e = 0; e < E; ++e) y[e] = apply(f, x0[u][e], x1[u][e], x2[u][e]);
      }
      EO::template store_vec<E>(a.data[0], base[0] + i, a.dtype[0], y);
    }
    return;
  }
  int valid[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t i = i0 + (int64_t)u * kBlock * E;
    const int64_t left = a.n0 - i;
    valid[u] = left >= E ? E : (left > 0 ? (int)left : 0);
    if (valid[u] > 0) {
      vec_fetch<typename F::In0, E, STREAM>(a, 1, base[1], i, valid[u], x0[u]);
      if constexpr (F::NIN >= 2) vec_fetch<typename F::In1, E, STREAM>(a, 2, base[2], i, valid[u], x1[u]);
      if constexpr (F::NIN >= 3) vec_fetch<typename F::In2, E, STREAM>(a, 3, base[3], i, valid[u], x2[u]);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (valid[u] == 0) continue;
    const int64_t i = i0 + (int64_t)u * kBlock * E;
    typename EO::value_t y[E];
#pragma unroll
    for (int e = 0; e < E; ++e) y[e] = apply(f, x0[u][e], x1[u][e], x2[u][e]);
    if (valid[u] == E) {
      EO::template store_vec<E>(a.data[0], base[0] + i, a.dtype[0], y);
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e)
        if (e < valid[u]) EO::store(a.data[0], base[0] + i + e, a.dtype[0], y[e]);
    }
  }
}

// Write-dominated broadcasts over a 2-D output (out[r][c] = f(a[r], b[c]) and the like: every input is constant along
// the inner dim, or along the outer dim, or both).  All the time goes into the stores, a workgroup moves one 4 KiB
// piece, and the pieces are handed out in address order so that the chip writes one sequential front; what is left
// to save is the workgroup's set-up, so this kernel takes a short argument block (one scalar load), one division, and
// static operand types.  [4096,1] + [1,4096] fp32: 11.0-11.3 us per launch against 12.3 us through ew_vec_kernel.
template <int NOPS> struct BcastArgs {
  char* data[NOPS];
  int64_t row_stride[NOPS];     // elements per outer step (inputs: 0 if constant along the outer dim)
  int inner[NOPS];              // inputs: 1 = follows the inner dim, 0 = constant along it
  FastDiv pieces_per_row;
};

template <class F, int E>
__global__ __launch_bounds__(kBlock) void ew_bcast_kernel(const F f, const BcastArgs<F::NIN + 1> a) {
  uint32_t row, piece;
  a.pieces_per_row.divmod(blockIdx.x, row, piece);
  const int64_t col = (int64_t)piece * (kBlock * E) + (int64_t)threadIdx.x * E;
  typename ValueOf<typename F::In0>::type x0[E];
  typename ValueOf<typename F::In1>::type x1[E];
  typename ValueOf<typename F::In2>::type x2[E];
  auto issue = [&](auto tag, int o, auto& x) {
    using In = typename decltype(tag)::type;
    if constexpr (!std::is_void<In>::value) {
      const int64_t base = (int64_t)row * a.row_stride[o];
      if (a.inner[o]) Elem<In>::template load_vec<E, false>(a.data[o], base + col, 0, x);
      else x[0] = Elem<In>::load(a.data[o], base, 0);
    }
  };
  auto spread = [&](auto tag, int o, auto& x) {
    using In = typename decltype(tag)::type;
    if constexpr (!std::is_void<In>::value) {
      if (!a.inner[o]) {
#pragma unroll
        for (int e = 1; e < E; ++e) x[e] = x[0];
      }
    }
  };
  issue(TypeTag<typename F::In0>{}, 1, x0);
  if constexpr (F::NIN >= 2) issue(TypeTag<typename F::In1>{}, 2, x1);
  if constexpr (F::NIN >= 3) issue(TypeTag<typename F::In2>{}, 3, x2);
  spread(TypeTag<typename F::In0>{}, 1, x0);
  if constexpr (F::NIN >= 2) spread(TypeTag<typename F::In1>{}, 2, x1);
  if constexpr (F::NIN >= 3) spread(TypeTag<typename F::In2>{}, 3, x2);
  using EO = Elem<typename F::Out>;
  typename EO::value_t y[E];
#pragma unroll
  for (int e = 0; e < E; ++e) y[e] = apply(f, x0[e], x1[e], x2[e]);
  EO::template store_vec<E>(a.data[0], (int64_t)row * a.row_stride[0] + col, 0, y);
}

// ---------------------------------------------------------------------------
// generic path
// ---------------------------------------------------------------------------
template <int NOPS> struct GenArgs {
  char* data[NOPS];
  int dtype[NOPS];
  int ndim;
  FastDiv fsize[TX_MAX_DIMS];
  int64_t size[TX_MAX_DIMS];
  int64_t stride[NOPS][TX_MAX_DIMS];
  int64_t numel;
};

template <class F, class IndexT, int U>
__global__ __launch_bounds__(kBlock) void ew_generic_kernel(const F f, const GenArgs<F::NIN + 1> a) {
  constexpr int NOPS = F::NIN + 1;
  const IndexT first = (IndexT)blockIdx.x * (kBlock * U) + threadIdx.x;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const IndexT lin = first + (IndexT)u * kBlock;
    if ((int64_t)lin >= a.numel) break;
    int64_t off[NOPS];
#pragma unroll
    for (int o = 0; o < NOPS; ++o) off[o] = 0;
    IndexT rem = lin;
    for (int d = a.ndim - 1; d >= 0; --d) {
      IndexT q, r;
      if constexpr (sizeof(IndexT) == 4) {
        a.fsize[d].divmod(rem, q, r);
      } else {
        q = rem / (IndexT)a.size[d];
        r = rem - q * (IndexT)a.size[d];
      }
      rem = q;
#pragma unroll
      for (int o = 0; o < NOPS; ++o) off[o] += (int64_t)r * a.stride[o][d];
    }
    typename ValueOf<typename F::In0>::type v0 = Elem<typename F::In0>::load(a.data[1], off[1], a.dtype[1]);
    typename ValueOf<typename F::In1>::type v1{};
    typename ValueOf<typename F::In2>::type v2{};
    if constexpr (F::NIN >= 2) v1 = Elem<typename F::In1>::load(a.data[2], off[2], a.dtype[2]);
    if constexpr (F::NIN >= 3) v2 = Elem<typename F::In2>::load(a.data[3], off[3], a.dtype[3]);
    Elem<typename F::Out>::store(a.data[0], off[0], a.dtype[0], apply(f, v0, v1, v2));
  }
}

// ---------------------------------------------------------------------------
// tile path: out[r][c] over a 2-D (optionally batched) problem where the
// output is contiguous along c and at least one input is contiguous along r.
// A 64x64 tile of each such input is read with lanes running along r, parked
// in LDS, and read back with lanes running along c.
// ---------------------------------------------------------------------------
// tile edge: 64 for value types up to 4 bytes, 32 for 8-byte values (keeps three staged operands inside 64 KB of LDS)
template <class F> constexpr int tile_edge() {
  return (sizeof(typename ValueOf<typename F::In0>::type) > 4 || sizeof(typename ValueOf<typename F::In1>::type) > 4 ||
          sizeof(typename ValueOf<typename F::In2>::type) > 4) ? 32 : 64;
}

template <int NOPS> struct TileArgs {
  char* data[NOPS];
  int dtype[NOPS];
  int64_t stride_r[NOPS], stride_c[NOPS], stride_b[NOPS];   // elements
  int transposed[NOPS];                                       // 1: stage through LDS
  int64_t rows, cols;
  FastDiv tiles_c, tiles_r;
};

template <class In, class V, int T, int NOPS>
__device__ __forceinline__ void tile_stage(const TileArgs<NOPS>& a, int o, int64_t boff, int64_t r0, int64_t c0,
                                           V (*lds)[T + 1]) {
  // lanes run along r (this operand's unit-stride dim): thread (tx, ty) reads row r0+tx, cols c0+ty+k*(256/T)
  constexpr int P = kBlock / T;
  const int tx = threadIdx.x % T, ty = threadIdx.x / T;
  const int64_t r = r0 + tx;
#pragma unroll 4
  for (int k = 0; k < T / P; ++k) {
    const int c = ty + P * k;
    if (r < a.rows && c0 + c < a.cols)
      lds[c][tx] = Elem<In>::load(a.data[o], boff + r * a.stride_r[o] + (c0 + c) * a.stride_c[o], a.dtype[o]);
  }
}

template <class In, class V, int T, int NOPS>
__device__ __forceinline__ V tile_fetch(const TileArgs<NOPS>& a, int o, int64_t boff, int64_t r, int64_t c, int lr,
                                        int lc, V (*lds)[T + 1]) {
  if (a.transposed[o]) return lds[lc][lr];
  return Elem<In>::load(a.data[o], boff + r * a.stride_r[o] + c * a.stride_c[o], a.dtype[o]);
}

template <class F>
__global__ __launch_bounds__(kBlock) void ew_tile_kernel(const F f, const TileArgs<F::NIN + 1> a) {
  constexpr int NOPS = F::NIN + 1;
  constexpr int kTile = tile_edge<F>();
  constexpr int P = kBlock / kTile;
  using V0 = typename ValueOf<typename F::In0>::type;
  using V1 = typename ValueOf<typename F::In1>::type;
  using V2 = typename ValueOf<typename F::In2>::type;
  __shared__ V0 l0[kTile][kTile + 1];
  __shared__ V1 l1[F::NIN >= 2 ? kTile : 1][kTile + 1];
  __shared__ V2 l2[F::NIN >= 3 ? kTile : 1][kTile + 1];
  uint32_t rest, tc, batch, tr;
  // Workgroups walk the tile grid along its diagonals: with a row pitch that is a multiple of the channel
  // interleave (8192 fp32 = 32 KiB), tiles of one tile-row read their transposed operand from the same HBM
  // channels, and tiles of one tile-column write to the same channels; neighbours on a diagonal share neither.
  a.tiles_r.divmod(blockIdx.x, rest, tr);
  a.tiles_c.divmod(rest, batch, tc);
  tc = (tc + tr) % a.tiles_c.d;
  const int64_t r0 = (int64_t)tr * kTile, c0 = (int64_t)tc * kTile;
  int64_t boff[NOPS];
#pragma unroll
  for (int o = 0; o < NOPS; ++o) boff[o] = (int64_t)batch * a.stride_b[o];
  if (a.transposed[1]) tile_stage<typename F::In0, V0, kTile>(a, 1, boff[1], r0, c0, l0);
  if constexpr (F::NIN >= 2)
    if (a.transposed[2]) tile_stage<typename F::In1, V1, kTile>(a, 2, boff[2], r0, c0, l1);
  if constexpr (F::NIN >= 3)
    if (a.transposed[3]) tile_stage<typename F::In2, V2, kTile>(a, 3, boff[3], r0, c0, l2);
  __syncthreads();
  // lanes run along c: thread (tx, ty) writes col c0+tx, rows r0+ty+k*(256/T)
  const int tx = threadIdx.x % kTile, ty = threadIdx.x / kTile;
  const int64_t c = c0 + tx;
#pragma unroll 4
  for (int k = 0; k < kTile / P; ++k) {
    const int lr = ty + P * k;
    const int64_t r = r0 + lr;
    if (r < a.rows && c < a.cols) {
      V0 v0 = tile_fetch<typename F::In0, V0, kTile>(a, 1, boff[1], r, c, lr, tx, l0);
      V1 v1{};
      V2 v2{};
      if constexpr (F::NIN >= 2) v1 = tile_fetch<typename F::In1, V1, kTile>(a, 2, boff[2], r, c, lr, tx, l1);
      if constexpr (F::NIN >= 3) v2 = tile_fetch<typename F::In2, V2, kTile>(a, 3, boff[3], r, c, lr, tx, l2);
      Elem<typename F::Out>::store(a.data[0], boff[0] + r * a.stride_r[0] + c * a.stride_c[0], a.dtype[0],
                                   apply(f, v0, v1, v2));
    }
  }
}

// Vectorised tile kernel for functors whose operands all have the same static element size S (2, 4 or
// 8 bytes): every global access is a 16-byte vector of V = 16/S elements.  A transposed operand is read
// with lanes along r (its unit-stride dim), written element-wise into a padded LDS tile, and read back
// transposed as V scalars per lane; the other operands and the output move as vectors along c.
template <class F> struct TileVec {
  static constexpr bool eligible =
      !Shape<F>::dynamic && Shape<F>::min_size == Shape<F>::max_size && Shape<F>::min_size >= 2 &&
      (F::NIN < 2 || static_size_of<typename F::In1>() == Shape<F>::min_size) &&
      (F::NIN < 3 || static_size_of<typename F::In2>() == Shape<F>::min_size);
  static constexpr int S = eligible ? Shape<F>::min_size : 4;
  static constexpr int V = 16 / S;
  static constexpr int T = S == 8 ? 32 : 64;            // tile edge in elements
  static constexpr int PITCH = T + (S >= 4 ? 1 : 4 / S);  // LDS row pitch (odd number of 4-byte words for S <= 4)
  static constexpr int LANES = T / V;                   // lanes that cover one tile row with vectors
  static constexpr int ROWS_PER_PASS = kBlock / LANES;
  static constexpr int PASSES = T / ROWS_PER_PASS;
};

// The three helpers below issue every global load of a tile unconditionally (positions outside the tensor are
// clamped onto its last vector and discarded later), so that all loads of a workgroup are in flight together:
// a load inside `if (in range)` is waited for inside that branch.
template <class In, class F, int NOPS>
__device__ __forceinline__ void tilev_stage_load(const TileArgs<NOPS>& a, int o, int64_t boff, int64_t r0, int64_t c0,
                                                 Vec<typename ValueOf<In>::type, TileVec<F>::V> (&t)[TileVec<F>::PASSES]) {
  using TV = TileVec<F>;
  using E = typename ValueOf<In>::type;
  const int rv = threadIdx.x % TV::LANES, cl = threadIdx.x / TV::LANES;
  const int64_t r = std::min<int64_t>(r0 + rv * TV::V, a.rows - TV::V);      // rows is a multiple of V on this path
#pragma unroll
  for (int k = 0; k < TV::PASSES; ++k) {
    const int64_t c = std::min<int64_t>(c0 + cl + TV::ROWS_PER_PASS * k, a.cols - 1);
    // cached loads: a 128-byte line of the transposed operand is consumed by several of these 16-byte accesses
    t[k] = vec_load<E, TV::V, false>((const E*)a.data[o] + boff + r + c * a.stride_c[o]);
  }
}
template <class In, class F, int NOPS>
__device__ __forceinline__ void tilev_stage_write(const TileArgs<NOPS>& a, int64_t r0, int64_t c0,
                                                  const Vec<typename ValueOf<In>::type, TileVec<F>::V> (&t)[TileVec<F>::PASSES],
                                                  typename ValueOf<In>::type* lds) {
  using TV = TileVec<F>;
  const int rv = threadIdx.x % TV::LANES, cl = threadIdx.x / TV::LANES;
  const bool row_ok = r0 + rv * TV::V < a.rows;
#pragma unroll
  for (int k = 0; k < TV::PASSES; ++k) {
    const int c = cl + TV::ROWS_PER_PASS * k;
    if (row_ok && c0 + c < a.cols) {
#pragma unroll
      for (int j = 0; j < TV::V; ++j) lds[c * TV::PITCH + rv * TV::V + j] = t[k].v[j];
    }
  }
}
// operands read along the output's fast dim (unit stride; the host sends anything else to the scalar tile kernel)
template <class In, class F, int NOPS>
__device__ __forceinline__ void tilev_straight_load(const TileArgs<NOPS>& a, int o, int64_t boff, int64_t r0, int64_t c0,
                                                    Vec<typename ValueOf<In>::type, TileVec<F>::V> (&g)[TileVec<F>::PASSES]) {
  using TV = TileVec<F>;
  using E = typename ValueOf<In>::type;
  const int cv = threadIdx.x % TV::LANES, rl = threadIdx.x / TV::LANES;
  const int64_t c = std::min<int64_t>(c0 + cv * TV::V, a.cols - TV::V);      // cols is a multiple of V on this path
  if (a.stride_c[o] == 0) {                    // constant along the output's fast dim (a column vector, a scalar): one element per row
#pragma unroll
    for (int k = 0; k < TV::PASSES; ++k) {
      const int64_t r = std::min<int64_t>(r0 + rl + TV::ROWS_PER_PASS * k, a.rows - 1);
      const E v = ((const E*)a.data[o])[boff + r * a.stride_r[o]];
#pragma unroll
      for (int j = 0; j < TV::V; ++j) g[k].v[j] = v;
    }
    return;
  }
#pragma unroll
  for (int k = 0; k < TV::PASSES; ++k) {
    const int64_t r = std::min<int64_t>(r0 + rl + TV::ROWS_PER_PASS * k, a.rows - 1);
    g[k] = vec_load<E, TV::V, false>((const E*)a.data[o] + boff + r * a.stride_r[o] + c);   // measured: the hint costs 10 % here
  }
}

// TMASK: bit i set = input i is the transposed one (compile-time, so that the loads of all operands form one
// straight-line group)
template <class F, int TMASK>
__global__ __launch_bounds__(kBlock) void ew_tile_vec_kernel(const F f, const TileArgs<F::NIN + 1> a) {
  using TV = TileVec<F>;
  constexpr int NOPS = F::NIN + 1;
  using V0 = typename ValueOf<typename F::In0>::type;
  using V1 = typename ValueOf<typename F::In1>::type;
  using V2 = typename ValueOf<typename F::In2>::type;
  using VO = typename ValueOf<typename F::Out>::type;
  // LDS only for the operands that are staged: an array per input whether transposed or not left a binary operator
  // with one transposed input half the resident workgroups of the transposed copy
  constexpr bool t0 = (TMASK & 1) != 0, t1 = (TMASK & 2) != 0, t2 = (TMASK & 4) != 0;
  __shared__ V0 l0[t0 ? TV::T * TV::PITCH : 1];
  __shared__ V1 l1[t1 ? TV::T * TV::PITCH : 1];
  __shared__ V2 l2[t2 ? TV::T * TV::PITCH : 1];
  uint32_t rest, tc, batch, tr;
  // diagonal walk over the tile grid (see ew_tile_kernel): 180 us -> 148 us for fp32 [8192,8192]
  a.tiles_r.divmod(blockIdx.x, rest, tr);
  a.tiles_c.divmod(rest, batch, tc);
  tc = (tc + tr) % a.tiles_c.d;
  const int64_t r0 = (int64_t)tr * TV::T, c0 = (int64_t)tc * TV::T;
  int64_t boff[NOPS];
#pragma unroll
  for (int o = 0; o < NOPS; ++o) boff[o] = (int64_t)batch * a.stride_b[o];
  // every global load of the tile first (a transposed operand lands in g* in its own orientation and goes
  // through LDS; the others are already laid out like the output), then LDS, then compute and store
  Vec<V0, TV::V> g0[TV::PASSES];
  Vec<V1, TV::V> g1[TV::PASSES];
  Vec<V2, TV::V> g2[TV::PASSES];
  if constexpr (t0) tilev_stage_load<typename F::In0, F>(a, 1, boff[1], r0, c0, g0);
  else tilev_straight_load<typename F::In0, F>(a, 1, boff[1], r0, c0, g0);
  if constexpr (F::NIN >= 2) {
    if constexpr (t1) tilev_stage_load<typename F::In1, F>(a, 2, boff[2], r0, c0, g1);
    else tilev_straight_load<typename F::In1, F>(a, 2, boff[2], r0, c0, g1);
  }
  if constexpr (F::NIN >= 3) {
    if constexpr (t2) tilev_stage_load<typename F::In2, F>(a, 3, boff[3], r0, c0, g2);
    else tilev_straight_load<typename F::In2, F>(a, 3, boff[3], r0, c0, g2);
  }
  if constexpr (t0) tilev_stage_write<typename F::In0, F>(a, r0, c0, g0, l0);
  if constexpr (F::NIN >= 2 && t1) tilev_stage_write<typename F::In1, F>(a, r0, c0, g1, l1);
  if constexpr (F::NIN >= 3 && t2) tilev_stage_write<typename F::In2, F>(a, r0, c0, g2, l2);
  __syncthreads();
  const int cv = threadIdx.x % TV::LANES, rl = threadIdx.x / TV::LANES;
  const int lc = cv * TV::V;
  const int64_t c = c0 + lc;
#pragma unroll
  for (int k = 0; k < TV::PASSES; ++k) {
    const int lr = rl + TV::ROWS_PER_PASS * k;
    const int64_t r = r0 + lr;
    V0 x0[TV::V];
    V1 x1[TV::V];
    V2 x2[TV::V];
#pragma unroll
    for (int j = 0; j < TV::V; ++j) {
      if constexpr (t0) x0[j] = l0[(lc + j) * TV::PITCH + lr];
      else x0[j] = g0[k].v[j];
      if constexpr (F::NIN < 2) x1[j] = V1();
      else if constexpr (t1) x1[j] = l1[(lc + j) * TV::PITCH + lr];
      else x1[j] = g1[k].v[j];
      if constexpr (F::NIN < 3) x2[j] = V2();
      else if constexpr (t2) x2[j] = l2[(lc + j) * TV::PITCH + lr];
      else x2[j] = g2[k].v[j];
    }
    if (r < a.rows && c < a.cols) {             // cols is a multiple of V on this path
      Vec<VO, TV::V> y;
#pragma unroll
      for (int j = 0; j < TV::V; ++j) y.v[j] = apply(f, x0[j], x1[j], x2[j]);
      vec_store<VO, TV::V, true>((VO*)a.data[0] + boff[0] + r * a.stride_r[0] + c, y);
    }
  }
}

// ---------------------------------------------------------------------------
// path selection + launch
// ---------------------------------------------------------------------------
inline bool aligned_to(const void* p, int bytes) { return ((uintptr_t)p % (uintptr_t)bytes) == 0; }

template <class F> bool vec_path_ok(const Iter& it, int E) {
  const int in = it.ndim - 1;
  if (it.op[0].stride[in] != 1 && it.size[in] != 1) return false;
  for (int o = 0; o < it.nops; ++o) {
    const int64_t s = it.op[o].stride[in];
    if (s != 0 && s != 1) return false;
    if (s == 1) {
      const int es = dtype_size(it.op[o].dtype);
      const int al = std::min(16, E * es);
      if (!aligned_to(it.op[o].data, al)) return false;
      for (int d = 0; d < in; ++d)
        if ((it.op[o].stride[d] * es) % al != 0) return false;
    }
  }
  int64_t outer = 1;
  for (int d = 0; d < in; ++d) outer *= it.size[d];
  const int64_t tile = (int64_t)kBlock * E * Shape<F>::U;
  const int64_t tiles = (it.size[in] + tile - 1) / tile;
  if (outer >= (1ll << 31) || tiles >= (1ll << 31) || outer * tiles >= (1ll << 31)) return false;
  return true;
}

// 2-D (+ batch) problem in which some input has unit stride along the output's outer dim
bool tile_path_ok(const Iter& it, int kTile) {
  if (it.ndim < 2 || it.ndim > 3) return false;
  const int c = it.ndim - 1, r = it.ndim - 2;
  if (it.op[0].stride[c] != 1) return false;
  bool any = false;
  for (int o = 1; o < it.nops; ++o)
    if (it.op[o].stride[r] == 1 && it.op[o].stride[c] != 1 && it.op[o].stride[c] != 0) any = true;
  if (!any) return false;
  const int64_t tr = (it.size[r] + kTile - 1) / kTile, tc = (it.size[c] + kTile - 1) / kTile;
  const int64_t nb = it.ndim == 3 ? it.size[0] : 1;
  return tr * tc < (1ll << 31) && tr * tc * nb < (1ll << 31);
}

template <class F> tx_status launch_ew(const Iter& it, const F& f, hipStream_t stream) {
  constexpr int NOPS = F::NIN + 1;
  constexpr int E = Shape<F>::E, U = Shape<F>::U;
  const char* forced = forced_path();
  const int in = it.ndim - 1;
  // run-time dtypes: the widest operand actually present sets the vector width (2 elements for 8-byte operands)
  int e_rt = E;
  if constexpr (Shape<F>::dynamic) {
    int widest = 1;
    for (int o = 0; o < it.nops; ++o) widest = std::max(widest, dtype_size(it.op[o].dtype));
    e_rt = widest >= 8 ? 2 : 4;
  }
  bool can_vec = vec_path_ok<F>(it, e_rt);
  constexpr int kTile = tile_edge<F>();
  bool can_tile = tile_path_ok(it, kTile);
  // automatic choice: vec unless rows are too short to fill a wave's worth of vectors
  bool use_vec = can_vec && (it.ndim == 1 || it.size[in] >= 64 * e_rt);
  bool use_tile = !use_vec && can_tile;
  if (!strcmp(forced, "vec") && can_vec) { use_vec = true; use_tile = false; }
  if (!strcmp(forced, "tile") && can_tile) { use_vec = false; use_tile = true; }
  if (!strcmp(forced, "generic")) { use_vec = false; use_tile = false; }

  if (use_vec) {
    VecArgs<NOPS> a;
    for (int o = 0; o < NOPS; ++o) {
      a.data[o] = it.op[o].data;
      a.dtype[o] = it.op[o].dtype;
      a.inner_stride[o] = (int)it.op[o].stride[in];
      a.stream[o] = a.inner_stride[o] == 1;
      for (int d = 0; d < in; ++d) {
        a.ostride[o][d] = it.op[o].stride[d];
        if (it.op[o].stride[d] == 0) a.stream[o] = 0;
      }
    }
    a.inner_stride[0] = 1;
    a.nouter = in;
    int64_t outer = 1;
    for (int d = 0; d < in; ++d) { a.osize[d] = FastDiv((uint32_t)it.size[d]); outer *= it.size[d]; }
    for (int d = in; d < TX_MAX_DIMS - 1; ++d) {         // unused outer dims: size 1, stride 0 (the kernel's unrolled part reads two)
      a.osize[d] = FastDiv(1);
      for (int o = 0; o < NOPS; ++o) a.ostride[o][d] = 0;
    }
    a.n0 = it.size[in];
    // write-dominated case (every input is a broadcast that stays in cache): four vectors per lane.  A workgroup's
    // lifetime is then dominated by its scalar set-up and one load round trip whatever it stores, and with one vector
    // per lane the [4096,1] + [1,4096] add needs 16384 such lifetimes (14.8 us per launch against 12.3 us with four,
    // graph replay so that the host's launch cost is out of the measurement; "vec-narrow" selects one vector)
    bool wide = !Shape<F>::dynamic && strcmp(forced, "vec-narrow") != 0;
    for (int o = 1; o < NOPS; ++o) wide = wide && !a.stream[o];
    constexpr int UW = 4;
    if constexpr (!Shape<F>::dynamic) {
      // the lean form: one outer dim, whole 4 KiB pieces, every input constant along at least one of the two dims
      bool lean = wide && in == 1 && a.n0 % (kBlock * E) == 0 && strcmp(forced, "vec-wide") != 0 && strcmp(forced, "vec-narrow") != 0;
      for (int o = 1; lean && o < NOPS; ++o) lean = a.inner_stride[o] == 0 || a.ostride[o][0] == 0;
      const int64_t pieces = a.n0 / (kBlock * E);
      if (lean && outer * pieces < (1ll << 31)) {
        BcastArgs<NOPS> b;
        for (int o = 0; o < NOPS; ++o) {
          b.data[o] = a.data[o];
          b.row_stride[o] = a.ostride[o][0];
          b.inner[o] = a.inner_stride[o];
        }
        b.pieces_per_row = FastDiv((uint32_t)pieces);
        set_path("vec-bcast");
        hipLaunchKernelGGL((ew_bcast_kernel<F, E>), dim3((unsigned)(outer * pieces)), dim3(kBlock), 0, stream, f, b);
        return check_launch("elementwise broadcast kernel");
      }
    }
    const int u_rt = wide ? UW : U;
    const int64_t tile = (int64_t)kBlock * e_rt * u_rt;
    const int64_t tiles = (a.n0 + tile - 1) / tile;
    if (outer * tiles >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "tensor too large for one launch");
    a.tiles_per_row = FastDiv((uint32_t)tiles);
    set_path("vec");
    const dim3 grid((unsigned)(outer * tiles));
    // all inputs streamed (a stride-0 inner operand is one scalar load and does not count)
    bool all_stream = strcmp(forced, "vec-cached") != 0;    // "vec-cached": plain loads, to measure what the hint is worth
    for (int o = 1; o < NOPS; ++o) all_stream = all_stream && (a.stream[o] || a.inner_stride[o] == 0);
    if constexpr (Shape<F>::dynamic) {
      if (e_rt == 2 && all_stream) hipLaunchKernelGGL((ew_vec_kernel<F, 2, U, true>), grid, dim3(kBlock), 0, stream, f, a);
      else if (e_rt == 2) hipLaunchKernelGGL((ew_vec_kernel<F, 2, U, false>), grid, dim3(kBlock), 0, stream, f, a);
      else if (all_stream) hipLaunchKernelGGL((ew_vec_kernel<F, 4, U, true>), grid, dim3(kBlock), 0, stream, f, a);
      else hipLaunchKernelGGL((ew_vec_kernel<F, 4, U, false>), grid, dim3(kBlock), 0, stream, f, a);
    } else {
      if (wide) hipLaunchKernelGGL((ew_vec_kernel<F, E, UW, false>), grid, dim3(kBlock), 0, stream, f, a);
      else if (all_stream) hipLaunchKernelGGL((ew_vec_kernel<F, E, U, true>), grid, dim3(kBlock), 0, stream, f, a);
      else hipLaunchKernelGGL((ew_vec_kernel<F, E, U, false>), grid, dim3(kBlock), 0, stream, f, a);
    }
    return check_launch("elementwise vec kernel");
  }
  if (use_tile) {
    TileArgs<NOPS> a;
    const int c = it.ndim - 1, r = it.ndim - 2;
    for (int o = 0; o < NOPS; ++o) {
      a.data[o] = it.op[o].data;
      a.dtype[o] = it.op[o].dtype;
      a.stride_r[o] = it.op[o].stride[r];
      a.stride_c[o] = it.op[o].stride[c];
      a.stride_b[o] = it.ndim == 3 ? it.op[o].stride[0] : 0;
      a.transposed[o] = o > 0 && a.stride_r[o] == 1 && a.stride_c[o] != 1 && a.stride_c[o] != 0;
    }
    a.rows = it.size[r];
    a.cols = it.size[c];
    if constexpr (TileVec<F>::eligible) {
      using TV = TileVec<F>;
      bool ok = a.rows % TV::V == 0 && a.cols % TV::V == 0;
      for (int o = 0; ok && o < NOPS; ++o) {
        if (o > 0 && a.stride_c[o] == 0 && !a.transposed[o]) continue;      // read as single elements: any alignment
        ok = aligned_to(a.data[o], 16) && (a.stride_b[o] * TV::S) % 16 == 0;
        if (a.transposed[o]) ok = ok && (a.stride_c[o] * TV::S) % 16 == 0;
        else if (a.stride_c[o] == 1) ok = ok && (a.stride_r[o] * TV::S) % 16 == 0;
        else ok = false;
      }
      const int64_t vtr = (a.rows + TV::T - 1) / TV::T, vtc = (a.cols + TV::T - 1) / TV::T;
      const int64_t vnb = it.ndim == 3 ? it.size[0] : 1;
      if (ok && vtr * vtc * vnb < (1ll << 31)) {
        a.tiles_c = FastDiv((uint32_t)vtc);
        a.tiles_r = FastDiv((uint32_t)vtr);
        set_path("tile");
        const dim3 vgrid((unsigned)(vtr * vtc * vnb));
        int mask = 0;
        for (int o = 1; o < NOPS; ++o) mask |= a.transposed[o] ? 1 << (o - 1) : 0;
        bool launched = true;
        switch (mask) {
          case 1: hipLaunchKernelGGL((ew_tile_vec_kernel<F, 1>), vgrid, dim3(kBlock), 0, stream, f, a); break;
          case 2: if constexpr (F::NIN >= 2) hipLaunchKernelGGL((ew_tile_vec_kernel<F, 2>), vgrid, dim3(kBlock), 0, stream, f, a); break;
          case 3: if constexpr (F::NIN >= 2) hipLaunchKernelGGL((ew_tile_vec_kernel<F, 3>), vgrid, dim3(kBlock), 0, stream, f, a); break;
          case 4: if constexpr (F::NIN >= 3) hipLaunchKernelGGL((ew_tile_vec_kernel<F, 4>), vgrid, dim3(kBlock), 0, stream, f, a); break;
          case 5: if constexpr (F::NIN >= 3) hipLaunchKernelGGL((ew_tile_vec_kernel<F, 5>), vgrid, dim3(kBlock), 0, stream, f, a); break;
          case 6: if constexpr (F::NIN >= 3) hipLaunchKernelGGL((ew_tile_vec_kernel<F, 6>), vgrid, dim3(kBlock), 0, stream, f, a); break;
          case 7: if constexpr (F::NIN >= 3) hipLaunchKernelGGL((ew_tile_vec_kernel<F, 7>), vgrid, dim3(kBlock), 0, stream, f, a); break;
          default: launched = false; break;    // no transposed input: not a tile problem
        }
        if (launched) {
          set_path("tile");
          return check_launch("elementwise vector tile kernel");
        }
      }
    }
    const int64_t tr = (a.rows + kTile - 1) / kTile, tc = (a.cols + kTile - 1) / kTile;
    const int64_t nb = it.ndim == 3 ? it.size[0] : 1;
    a.tiles_c = FastDiv((uint32_t)tc);
    a.tiles_r = FastDiv((uint32_t)tr);
    set_path("tile-scalar");
    hipLaunchKernelGGL((ew_tile_kernel<F>), dim3((unsigned)(tr * tc * nb)), dim3(kBlock), 0, stream, f, a);
    return check_launch("elementwise tile kernel");
  }
  GenArgs<NOPS> a;
  for (int o = 0; o < NOPS; ++o) {
    a.data[o] = it.op[o].data;
    a.dtype[o] = it.op[o].dtype;
    for (int d = 0; d < it.ndim; ++d) a.stride[o][d] = it.op[o].stride[d];
  }
  a.ndim = it.ndim;
  a.numel = it.numel;
  bool small = it.numel < (1ll << 31);
  for (int d = 0; d < it.ndim; ++d) {
    a.size[d] = it.size[d];
    a.fsize[d] = FastDiv((uint32_t)std::min<int64_t>(it.size[d], 0x7fffffff));
  }
  constexpr int GU = 4;
  const int64_t per_block = (int64_t)kBlock * GU;
  const int64_t blocks = (it.numel + per_block - 1) / per_block;
  if (blocks >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "tensor too large for the generic elementwise path");
  set_path("generic");
  if (small)
    hipLaunchKernelGGL((ew_generic_kernel<F, uint32_t, GU>), dim3((unsigned)blocks), dim3(kBlock), 0, stream, f, a);
  else
    hipLaunchKernelGGL((ew_generic_kernel<F, uint64_t, GU>), dim3((unsigned)blocks), dim3(kBlock), 0, stream, f, a);
  return check_launch("elementwise generic kernel");
}

// ---------------------------------------------------------------------------
// functors
// ---------------------------------------------------------------------------
// round a float to the common half dtype and back (identity for fp32)
__device__ __forceinline__ float quantize(float v, int common) {
  if (common == TX_BF16) return bf16_to_float(float_to_bf16(v));
  if (common == TX_F16) return (float)(f16)v;
  return v;
}

// run(): fp32 result within 2 ulp.  run_half(): for fp16 / bf16 results, which are rounded to 8-11 bits
// anyway, plain fp32 compositions are accurate enough and several times cheaper than the binary64 forms.
struct OpExp {
  __device__ static float run(float x) { return expf(x); }
  __device__ static float run_half(float x) { return expf(x); }
};
struct OpLog {
  __device__ static float run(float x) { return logf(x); }
  __device__ static float run_half(float x) { return logf(x); }
};
struct OpSqrt {
  __device__ static float run(float x) { return sqrtf(x); }
  __device__ static float run_half(float x) { return sqrtf(x); }
};
struct OpSigmoid {
  static constexpr int VPL = 2;
  __device__ static float run(float x) { return sigmoid_f32(x); }
  __device__ static float run_half(float x) { return 1.0f / (1.0f + expf(-x)); }
};
struct OpTanh {
  static constexpr int VPL = 2;
  __device__ static float run(float x) { return tanh_f32(x); }
  __device__ static float run_half(float x) { return tanhf(x); }
};
struct OpGelu {
  static constexpr int VPL = 2;
  __device__ static float run(float x) { return gelu_erf_f32(x); }
  template <int N> __device__ static void run_n(const float (&x)[N], float (&y)[N]) {
    const GeluLead k = gelu_lead();
#pragma unroll
    for (int i = 0; i < N; ++i) y[i] = gelu_erf_f32(x[i], k);
  }
  // x * erfc(-x / sqrt 2) / 2: erfc keeps its relative accuracy in the negative tail
  __device__ static float run_half(float x) { return gelu_erf_half(x); }
};

struct OpLog1p {
  static constexpr int VPL = 2;
  __device__ static float run(float x) { return log1p_f32(x); }
  __device__ static float run_half(float x) { return log1pf(x); }
};
struct OpExpm1 {
  __device__ static float run(float x) { return expm1f(x); }
  __device__ static float run_half(float x) { return expm1f(x); }
};
// log(sigmoid(x)) = min(x, 0) - log1p(exp(-|x|)): neither tail overflows or cancels
struct OpLogSigmoid {
  static constexpr int VPL = 2;
  __device__ static float run(float x) { return logsigmoid_f32(x); }
  __device__ static float run_half(float x) { return logsigmoid_half(x); }
};

enum { kAdd = TX_ADD, kMul = TX_MUL, kDiv = TX_DIV, kMax = TX_MAXIMUM, kEq = TX_EQ };

__device__ __forceinline__ float fmax_nan(float a, float b) {
  return (a != a || b != b) ? __uint_as_float(0x7fc00000u) : (b > a ? b : a);
}
__device__ __forceinline__ float fmin_nan(float a, float b) {
  return (a != a || b != b) ? __uint_as_float(0x7fc00000u) : (b < a ? b : a);
}
// the comparison and logical families, selected at run time (wave-uniform): one set of kernels serves all six
template <class V> __device__ __forceinline__ uint8_t compare(int code, V a, V b) {
  switch (code) {
    case TX_EQ: return a == b;
    case TX_NE: return a != b;
    case TX_LT: return a < b;
    case TX_LE: return a <= b;
    case TX_GT: return a > b;
    case TX_GE: return a >= b;
    case TX_LOGICAL_AND: return (a != V(0)) & (b != V(0));      // a NaN is not zero
    case TX_LOGICAL_OR: return (a != V(0)) | (b != V(0));
    default: return (a != V(0)) != (b != V(0));
  }
}


}  // namespace
}  // namespace tx
