// Shared host/device helpers of the gfx950 operator library (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/txops.h"

namespace tx {

// ---------------------------------------------------------------------------
// dtype helpers (host + device)
// ---------------------------------------------------------------------------
__host__ __device__ inline int dtype_size(int dt) {
  switch (dt) {
    case TX_BOOL: return 1;
    case TX_I32: return 4;
    case TX_I64: return 8;
    case TX_F16: return 2;
    case TX_BF16: return 2;
    case TX_F32: return 4;
  }
  return 0;
}
inline bool dtype_valid(int dt) { return dt >= TX_BOOL && dt <= TX_F32; }
inline int dtype_category(int dt) { return dt == TX_BOOL ? 0 : (dt <= TX_I64 ? 1 : 2); }
inline bool dtype_is_float(int dt) { return dt >= TX_F16; }
inline bool dtype_is_half(int dt) { return dt == TX_F16 || dt == TX_BF16; }
// may a result of dtype `from` be written to a tensor of dtype `to`: not a floating value into an integer or
// bool tensor, not an integer into a bool tensor
inline bool can_cast(int from, int to) {
  return !(dtype_is_float(from) && !dtype_is_float(to)) && !(from != TX_BOOL && to == TX_BOOL);
}
const char* dtype_name(int dt);

// ---------------------------------------------------------------------------
// host-side error reporting
// ---------------------------------------------------------------------------
tx_status fail(tx_status code, const char* fmt, ...);   // records the thread-local message, returns code
void set_path(const char* name);                         // records the dispatched kernel path
const char* forced_path();                               // "" when automatic
tx_status check_launch(const char* what);                // hipGetLastError -> TX_ERR_LAUNCH
// Header of a look-back workspace (single-pass scans, single-pass compaction): word 0 = ticket counter (low half) and
// error flag (high half, set when a bounded wait gave up), word 1 = this tag, written by the clearing kernel.
constexpr unsigned long long kLookbackMagic = 0x74784c6f6f6b6261ull;
// Index validation (validate.hip): whether the calling thread asked for it, and the pass itself - range-checks every
// value of `index` against [lo, hi) on the stream, synchronises it, and returns TX_OK or TX_ERR_INDEX.
bool index_validation_on();
tx_status validate_index(const tx_tensor* index, int64_t lo, int64_t hi, const char* what, hipStream_t stream);

tx_status check_tensor(const tx_tensor* t, const char* name);
inline int64_t numel(const tx_tensor* t) {
  int64_t n = 1;
  for (int d = 0; d < t->ndim; ++d) n *= t->sizes[d];
  return n;
}
bool same_sizes(const tx_tensor* t, int nd, const int64_t* sizes);
// wrap a possibly negative dim for a tensor of rank nd (rank 0 accepts 0 / -1)
tx_status wrap_dim(int64_t dim, int nd, int* out);

// promotion
int promote2(int a, int b);
int result_type(const tx_tensor* const* ops, int n);
tx_status broadcast_shapes(const tx_tensor* const* ops, int n, int* ndim, int64_t* sizes);

// Memory extent [lo, hi) in bytes covered by a tensor (empty tensors: lo == hi).
void byte_extent(const tx_tensor* t, uintptr_t* lo, uintptr_t* hi);
// true if the tensor's elements are all at distinct addresses (conservative: sorted-stride test)
bool no_internal_overlap(const tx_tensor* t);
// out vs. input aliasing rule: identical view is fine, disjoint is fine, anything else is overlap
bool partial_overlap(const tx_tensor* out, const tx_tensor* in);

// ---------------------------------------------------------------------------
// device element types
// ---------------------------------------------------------------------------
using f16 = _Float16;
struct bf16 {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_to_float(bf16 h) { return __uint_as_float(((uint32_t)h.bits) << 16); }
// round-to-nearest-even fp32 -> bf16; NaN stays NaN (quiet)
// (gfx950 has a hardware conversion; the compiler selects it for the __bf16 cast)
__device__ __forceinline__ bf16 float_to_bf16(float f) {
  bf16 r;
  r.bits = __builtin_bit_cast(uint16_t, (__bf16)f);
  return r;
}

template <class T> struct TypeTag;
template <> struct TypeTag<uint8_t> { static constexpr int value = TX_BOOL; };
template <> struct TypeTag<int32_t> { static constexpr int value = TX_I32; };
template <> struct TypeTag<int64_t> { static constexpr int value = TX_I64; };
template <> struct TypeTag<f16> { static constexpr int value = TX_F16; };
template <> struct TypeTag<bf16> { static constexpr int value = TX_BF16; };
template <> struct TypeTag<float> { static constexpr int value = TX_F32; };

// conversions between storage types and compute types
template <class To, class From> struct Cvt {
  __device__ __forceinline__ static To run(From v) { return (To)v; }
};
template <class T> struct Cvt<T, T> {
  __device__ __forceinline__ static T run(T v) { return v; }
};
template <> struct Cvt<float, bf16> {
  __device__ __forceinline__ static float run(bf16 v) { return bf16_to_float(v); }
};
template <> struct Cvt<bf16, float> {
  __device__ __forceinline__ static bf16 run(float v) { return float_to_bf16(v); }
};
template <> struct Cvt<double, bf16> {
  __device__ __forceinline__ static double run(bf16 v) { return (double)bf16_to_float(v); }
};
template <> struct Cvt<float, f16> {
  __device__ __forceinline__ static float run(f16 v) { return (float)v; }
};
template <> struct Cvt<f16, float> {
  __device__ __forceinline__ static f16 run(float v) { return (f16)v; }
};
// int64 -> half types goes through fp32 (nearest-even), like the conversion to the common dtype
template <> struct Cvt<bf16, int64_t> {
  __device__ __forceinline__ static bf16 run(int64_t v) { return float_to_bf16((float)v); }
};
template <> struct Cvt<bf16, double> {
  __device__ __forceinline__ static bf16 run(double v) { return float_to_bf16((float)v); }
};
template <> struct Cvt<uint8_t, float> {
  __device__ __forceinline__ static uint8_t run(float v) { return v != 0.0f; }
};
template <> struct Cvt<uint8_t, int64_t> {
  __device__ __forceinline__ static uint8_t run(int64_t v) { return v != 0; }
};
template <class To, class From> __device__ __forceinline__ To cvt(From v) { return Cvt<To, From>::run(v); }

// ---------------------------------------------------------------------------
// aligned vectors: N elements moved with the widest instruction that fits
// ---------------------------------------------------------------------------
template <int BYTES> struct VecAlign { static constexpr int value = BYTES >= 16 ? 16 : BYTES; };
template <class T, int N> struct alignas(VecAlign<sizeof(T) * N>::value) Vec {
  T v[N];
};

// Whole-vector loads and stores.  `nt` marks the access as streaming (non-temporal): data that is touched once
// should not displace lines other kernels may still want.  The access is made with a vector of the element's
// own machine type: when the bytes are loaded as integers and re-typed afterwards, the optimiser rewrites the
// load with the final type and the non-temporal hint is lost on the way.  NT is a template parameter for the
// same reason: a hint that depends on a run-time value (or on a function argument, before inlining) is
// dropped when the optimiser merges the two branches.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <class T> struct NativeElem { using type = T; };
template <> struct NativeElem<bf16> { using type = uint16_t; };
template <class T, int N> struct NativeVec {
  typedef typename NativeElem<T>::type type __attribute__((ext_vector_type(N)));
};

template <class T, int N, bool NT> __device__ __forceinline__ Vec<T, N> vec_load(const T* p) {
  using E = typename NativeElem<T>::type;
  constexpr int BYTES = sizeof(T) * N;
  static_assert(BYTES <= 16 || BYTES % 16 == 0, "vectors longer than 16 bytes are moved in 16-byte pieces");
  constexpr int M = BYTES > 16 ? 16 / (int)sizeof(T) : N;       // elements per access
  Vec<T, N> r;
  if constexpr (M == 1) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const E* q = (const E*)p + i;
      E c;
      if constexpr (NT) c = __builtin_nontemporal_load(q); else c = *q;
      r.v[i] = __builtin_bit_cast(T, c);
    }
  } else {
    using NV = typename NativeVec<T, M>::type;
#pragma unroll
    for (int i = 0; i < N / M; ++i) {
      const NV* q = (const NV*)p + i;
      NV c;
      if constexpr (NT) c = __builtin_nontemporal_load(q); else c = *q;
#pragma unroll
      for (int e = 0; e < M; ++e) r.v[i * M + e] = __builtin_bit_cast(T, (E)c[e]);
    }
  }
  return r;
}
template <class T, int N, bool NT> __device__ __forceinline__ void vec_store(T* p, const Vec<T, N>& v) {
  using E = typename NativeElem<T>::type;
  constexpr int BYTES = sizeof(T) * N;
  static_assert(BYTES <= 16 || BYTES % 16 == 0, "vectors longer than 16 bytes are moved in 16-byte pieces");
  constexpr int M = BYTES > 16 ? 16 / (int)sizeof(T) : N;
  if constexpr (M == 1) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      E* q = (E*)p + i;
      const E c = __builtin_bit_cast(E, v.v[i]);
      if constexpr (NT) __builtin_nontemporal_store(c, q); else *q = c;
    }
  } else {
    using NV = typename NativeVec<T, M>::type;
#pragma unroll
    for (int i = 0; i < N / M; ++i) {
      NV c;
#pragma unroll
      for (int e = 0; e < M; ++e) c[e] = __builtin_bit_cast(E, v.v[i * M + e]);
      NV* q = (NV*)p + i;
      if constexpr (NT) __builtin_nontemporal_store(c, q); else *q = c;
    }
  }
}

// ---------------------------------------------------------------------------
// division by a run-time constant (32-bit dividends), magic-number form:
// q = (n * m) >> (32 + s) with m = ceil(2^(32+s) / d), valid for n < 2^31
// ---------------------------------------------------------------------------
struct FastDiv {
  uint32_t d, m, s;
  FastDiv() : d(1), m(0), s(0) {}
  explicit FastDiv(uint32_t div) : d(div ? div : 1) {
    if (d == 1) { m = 0; s = 0; return; }
    s = 0;
    while ((1ull << s) < d) ++s;                       // s = ceil(log2 d)
    m = (uint32_t)(((1ull << 32) * ((1ull << s) - d)) / d + 1);
  }
  __host__ __device__ __forceinline__ uint32_t div(uint32_t n) const {   // d == 1: m = 0, s = 0 gives n without a branch
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t t = __umulhi(n, m);
#else
    uint32_t t = (uint32_t)(((uint64_t)n * m) >> 32);
#endif
    return (t + n) >> s;                                // n < 2^31 keeps t + n from wrapping
  }
  __host__ __device__ __forceinline__ void divmod(uint32_t n, uint32_t& q, uint32_t& r) const {
    q = div(n);
    r = n - q * d;
  }
};

// ---------------------------------------------------------------------------
// wave64 helpers
// ---------------------------------------------------------------------------
constexpr int kWave = 64;

template <class T> __device__ __forceinline__ T shfl_xor(T v, int mask) {
  static_assert(sizeof(T) == 4 || sizeof(T) == 8, "4- or 8-byte shuffles");
  if constexpr (sizeof(T) == 4) {
    int x = __builtin_bit_cast(int, v);
    x = __shfl_xor(x, mask, kWave);
    return __builtin_bit_cast(T, x);
  } else {
    long long x = __builtin_bit_cast(long long, v);
    x = __shfl_xor(x, mask, kWave);
    return __builtin_bit_cast(T, x);
  }
}
template <class T> __device__ __forceinline__ T shfl_up(T v, int delta) {
  if constexpr (sizeof(T) == 4) {
    int x = __builtin_bit_cast(int, v);
    x = __shfl_up(x, delta, kWave);
    return __builtin_bit_cast(T, x);
  } else {
    long long x = __builtin_bit_cast(long long, v);
    x = __shfl_up(x, delta, kWave);
    return __builtin_bit_cast(T, x);
  }
}
template <class T> __device__ __forceinline__ T shfl_idx(T v, int lane) {
  if constexpr (sizeof(T) == 4) {
    int x = __builtin_bit_cast(int, v);
    x = __shfl(x, lane, kWave);
    return __builtin_bit_cast(T, x);
  } else {
    long long x = __builtin_bit_cast(long long, v);
    x = __shfl(x, lane, kWave);
    return __builtin_bit_cast(T, x);
  }
}

inline hipStream_t as_stream(void* s) { return (hipStream_t)s; }

}  // namespace tx
