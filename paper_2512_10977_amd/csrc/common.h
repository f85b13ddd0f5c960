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
const char* dtype_name(int dt);

// ---------------------------------------------------------------------------
// host-side error reporting
// ---------------------------------------------------------------------------
tx_status fail(tx_status code, const char* fmt, ...);   // records the thread-local message, returns code
void set_path(const char* name);                         // records the dispatched kernel path
const char* forced_path();                               // "" when automatic
tx_status check_launch(const char* what);                // hipGetLastError -> TX_ERR_LAUNCH

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

// Whole-vector loads and stores.  `nt` marks the access as streaming (non-temporal):
// data that is touched once should not displace lines other kernels may still want.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <class T, int N> __device__ __forceinline__ Vec<T, N> vec_load(const T* p, bool nt) {
  constexpr int BYTES = sizeof(T) * N;
  Vec<T, N> r;
  if constexpr (BYTES % 16 == 0) {
#pragma unroll
    for (int i = 0; i < BYTES / 16; ++i) {
      const u32x4* q = (const u32x4*)p + i;
      u32x4 c = nt ? __builtin_nontemporal_load(q) : *q;
      __builtin_memcpy((char*)&r + 16 * i, &c, 16);
    }
  } else if constexpr (BYTES == 8) {
    const u32x2* q = (const u32x2*)p;
    u32x2 c = nt ? __builtin_nontemporal_load(q) : *q;
    __builtin_memcpy(&r, &c, 8);
  } else if constexpr (BYTES == 4) {
    const uint32_t* q = (const uint32_t*)p;
    uint32_t c = nt ? __builtin_nontemporal_load(q) : *q;
    __builtin_memcpy(&r, &c, 4);
  } else {
    r = *(const Vec<T, N>*)p;
  }
  return r;
}
template <class T, int N> __device__ __forceinline__ void vec_store(T* p, const Vec<T, N>& v, bool nt) {
  constexpr int BYTES = sizeof(T) * N;
  if constexpr (BYTES % 16 == 0) {
#pragma unroll
    for (int i = 0; i < BYTES / 16; ++i) {
      u32x4 c;
      __builtin_memcpy(&c, (const char*)&v + 16 * i, 16);
      u32x4* q = (u32x4*)p + i;
      if (nt) __builtin_nontemporal_store(c, q); else *q = c;
    }
  } else if constexpr (BYTES == 8) {
    u32x2 c;
    __builtin_memcpy(&c, &v, 8);
    if (nt) __builtin_nontemporal_store(c, (u32x2*)p); else *(u32x2*)p = c;
  } else if constexpr (BYTES == 4) {
    uint32_t c;
    __builtin_memcpy(&c, &v, 4);
    if (nt) __builtin_nontemporal_store(c, (uint32_t*)p); else *(uint32_t*)p = c;
  } else {
    *(Vec<T, N>*)p = v;
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
  __host__ __device__ __forceinline__ uint32_t div(uint32_t n) const {
    if (d == 1) return n;
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
