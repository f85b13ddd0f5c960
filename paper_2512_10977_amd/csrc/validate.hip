// Optional index validation: one extra pass over an index tensor, ahead of the data kernels, that range-checks
// every value and lets the host return TX_ERR_INDEX instead of launching a kernel that would read or write out of
// bounds.  Off by default (the pass ends in a stream synchronisation); switched on per calling thread with
// tx_set_index_validation, or for every thread from the start with the environment variable TX_VALIDATE_INDICES=1.
#include <cstdlib>
#include <mutex>

#include "common.h"

namespace tx {
namespace {

struct CheckArgs {
  const char* index;
  int is64;
  int ndim;
  int64_t size[TX_MAX_DIMS];
  int64_t stride_[TX_MAX_DIMS];
  int64_t numel;
  int64_t lo, hi;                       // valid values: lo <= v < hi
};

constexpr int kBlock = 256;
constexpr unsigned long long kNoBad = ~0ull;

// first[0]: smallest linear position (over the dims that are not repeats) of a value outside [lo, hi); kNoBad if none
__global__ __launch_bounds__(kBlock) void index_check_kernel(const CheckArgs a, unsigned long long* first) {
  const int64_t step = (int64_t)gridDim.x * kBlock;
  for (int64_t lin = (int64_t)blockIdx.x * kBlock + threadIdx.x; lin < a.numel; lin += step) {
    int64_t rem = lin, off = 0;
    for (int d = a.ndim - 1; d >= 0; --d) {
      const int64_t q = rem / a.size[d];
      off += (rem - q * a.size[d]) * a.stride_[d];
      rem = q;
    }
    const int64_t v = a.is64 ? ((const int64_t*)a.index)[off] : (int64_t)((const int32_t*)a.index)[off];
    if (v < a.lo || v >= a.hi) atomicMin(first, (unsigned long long)lin);   // the smallest offending position wins
  }
}
__global__ void index_check_clear_kernel(unsigned long long* first) { first[0] = kNoBad; }

// The flag word lives in the library image (one copy per GPU): the library allocates no device memory.
__device__ __align__(256) unsigned long long index_flag[32];
constexpr int kMaxDevices = 64;
std::mutex g_mutex;                       // one validation at a time: every call on a GPU shares that GPU's flag word
unsigned long long* g_flag_ptr[kMaxDevices] = {nullptr};

thread_local int t_validate = -1;         // -1: not set by this thread yet, take the environment's word

}  // namespace

bool index_validation_on() {
  if (t_validate < 0) {
    const char* e = std::getenv("TX_VALIDATE_INDICES");
    t_validate = (e && e[0] && !(e[0] == '0' && e[1] == 0)) ? 1 : 0;
  }
  return t_validate == 1;
}

tx_status validate_index(const tx_tensor* index, int64_t lo, int64_t hi, const char* what, hipStream_t s) {
  CheckArgs a;
  a.index = (const char*)index->data;
  a.is64 = index->dtype == TX_I64;
  a.ndim = 0;
  a.numel = 1;
  for (int d = 0; d < index->ndim; ++d) {
    if (index->sizes[d] == 0) return TX_OK;
    if (index->sizes[d] == 1 || index->strides[d] == 0) continue;     // a broadcast dim repeats values already checked
    a.size[a.ndim] = index->sizes[d];
    a.stride_[a.ndim] = index->strides[d];
    a.numel *= index->sizes[d];
    ++a.ndim;
  }
  a.lo = lo;
  a.hi = hi;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(TX_ERR_LAUNCH, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(TX_ERR_LAUNCH, "device ordinal %d is outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_flag_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(index_flag));
    if (e != hipSuccess || !p) return fail(TX_ERR_LAUNCH, "hipGetSymbolAddress(index_flag): %s", hipGetErrorString(e));
    g_flag_ptr[dev] = (unsigned long long*)p;
  }
  unsigned long long* flag = g_flag_ptr[dev];
  hipLaunchKernelGGL(index_check_clear_kernel, dim3(1), dim3(1), 0, s, flag);
  const int64_t blocks = std::min<int64_t>((a.numel + kBlock - 1) / kBlock, 4096);
  hipLaunchKernelGGL(index_check_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, a, flag);
  tx_status rc = check_launch("index validation kernel");
  if (rc) return rc;
  unsigned long long first = kNoBad;
  e = hipMemcpyAsync(&first, flag, sizeof(first), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail(TX_ERR_LAUNCH, "index validation: %s", hipGetErrorString(e));
  if (first == kNoBad) return TX_OK;
  // the offending value, for the message: one more small copy from the index tensor
  int64_t rem = (int64_t)first, off = 0;
  for (int d = a.ndim - 1; d >= 0; --d) {
    off += (rem % a.size[d]) * a.stride_[d];
    rem /= a.size[d];
  }
  long long value = 0;
  if (a.is64) {
    int64_t v = 0;
    if (hipMemcpy(&v, (const int64_t*)a.index + off, sizeof(v), hipMemcpyDeviceToHost) == hipSuccess) value = v;
  } else {
    int32_t v = 0;
    if (hipMemcpy(&v, (const int32_t*)a.index + off, sizeof(v), hipMemcpyDeviceToHost) == hipSuccess) value = v;
  }
  return fail(TX_ERR_INDEX, "%s: index value %lld (element offset %lld of the index tensor) is outside [%lld, %lld)", what,
              value, (long long)off, (long long)lo, (long long)hi);
}

}  // namespace tx

extern "C" {

tx_status tx_lookback_status(const void* ws, void* stream) {
  if (!ws) return tx::fail(TX_ERR_NULL, "tx_lookback_status: null workspace");
  unsigned long long head[2] = {0, 0};
  hipStream_t s = tx::as_stream(stream);
  hipError_t e = hipMemcpyAsync(head, ws, sizeof(head), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return tx::fail(TX_ERR_LAUNCH, "tx_lookback_status: %s", hipGetErrorString(e));
  if (head[1] != tx::kLookbackMagic) return TX_OK;               // not written by a look-back path: nothing to report
  if ((unsigned int)(head[0] >> 32) != 0)
    return tx::fail(TX_ERR_LAUNCH, "a look-back wait gave up (a predecessor tile never published its status); the output "
                                   "of the call that used this workspace is not valid");
  return TX_OK;
}

void tx_set_index_validation(int on) { tx::t_validate = on ? 1 : 0; }
int tx_get_index_validation(void) { return tx::index_validation_on() ? 1 : 0; }

}  // extern "C"
