// Instantiates the nansum / nanmean / count_nonzero / vector-norm reduction policies.
#include "reduce_impl.h"

namespace tx {
namespace red {

#define TX_FLOAT_DTYPES(...)                                                           \
  switch (x->dtype) {                                                                  \
    case TX_F32: return launch<__VA_ARGS__(float)>(p, x, out, c, ws, wsb, s);           \
    case TX_BF16: return launch<__VA_ARGS__(bf16)>(p, x, out, c, ws, wsb, s);           \
    case TX_F16: return launch<__VA_ARGS__(f16)>(p, x, out, c, ws, wsb, s);             \
    default: break;                                                                    \
  }

tx_status launch_nansum(bool mean, const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                        hipStream_t s) {
#define TX_NANMEAN(T) NanSumPolicy<T, true>
#define TX_NANSUM(T) NanSumPolicy<T, false>
  if (mean) {
    TX_FLOAT_DTYPES(TX_NANMEAN)
    return fail(TX_ERR_DTYPE, "nanmean takes floating dtypes only");
  }
  TX_FLOAT_DTYPES(TX_NANSUM)
  return launch_sum(false, p, x, out, c, ws, wsb, s);           // integers have no NaN
}

tx_status launch_count(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                       hipStream_t s) {
#define TX_COUNT(T) CountPolicy<T>
  TX_FLOAT_DTYPES(TX_COUNT)
  switch (x->dtype) {
    case TX_I64: return launch<CountPolicy<int64_t>>(p, x, out, c, ws, wsb, s);
    case TX_I32: return launch<CountPolicy<int32_t>>(p, x, out, c, ws, wsb, s);
    default: return launch<CountPolicy<uint8_t>>(p, x, out, c, ws, wsb, s);
  }
}

tx_status launch_norm(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                      hipStream_t s) {
#define TX_NORM0(T) NormPolicy<T, 0>
#define TX_NORM1(T) NormPolicy<T, 1>
#define TX_NORM2(T) NormPolicy<T, 2>
#define TX_NORM3(T) NormPolicy<T, 3>
#define TX_NORM4(T) NormPolicy<T, 4>
#define TX_NORM5(T) NormPolicy<T, 5>
  if (c == 0.0) { TX_FLOAT_DTYPES(TX_NORM0) }
  else if (c == 1.0) { TX_FLOAT_DTYPES(TX_NORM1) }
  else if (c == 2.0) { TX_FLOAT_DTYPES(TX_NORM2) }
  else if (c == __builtin_inf()) { TX_FLOAT_DTYPES(TX_NORM3) }
  else if (c == -__builtin_inf()) { TX_FLOAT_DTYPES(TX_NORM4) }
  else { TX_FLOAT_DTYPES(TX_NORM5) }
  return fail(TX_ERR_DTYPE, "norm takes floating dtypes only");
}

}  // namespace red
}  // namespace tx
