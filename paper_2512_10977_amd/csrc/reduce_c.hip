// Instantiates the amin / argmin / any / all / logsumexp reduction policies.
#include "reduce_impl.h"

namespace tx {
namespace red {

template <class T> using AminPolicy = AmaxPolicy<T, true>;
template <class T> using ArgminPolicy = ArgmaxPolicy<T, true>;

#define TX_ALL_DTYPES(POLICY)                                                          \
  switch (x->dtype) {                                                                  \
    case TX_F32: return launch<POLICY<float>>(p, x, out, c, ws, wsb, s);                \
    case TX_BF16: return launch<POLICY<bf16>>(p, x, out, c, ws, wsb, s);                \
    case TX_F16: return launch<POLICY<f16>>(p, x, out, c, ws, wsb, s);                  \
    case TX_I64: return launch<POLICY<int64_t>>(p, x, out, c, ws, wsb, s);              \
    case TX_I32: return launch<POLICY<int32_t>>(p, x, out, c, ws, wsb, s);              \
    default: break;                                                                    \
  }

tx_status launch_amin(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                      hipStream_t s) {
  TX_ALL_DTYPES(AminPolicy)
  return launch<AminPolicy<uint8_t>>(p, x, out, c, ws, wsb, s);
}

tx_status launch_argmin(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                        hipStream_t s) {
  TX_ALL_DTYPES(ArgminPolicy)
  return fail(TX_ERR_DTYPE, "argmin does not take bool");
}

tx_status launch_anyall(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                        hipStream_t s) {
  TX_ALL_DTYPES(AnyAllPolicy)
  return launch<AnyAllPolicy<uint8_t>>(p, x, out, c, ws, wsb, s);
}

tx_status launch_logsumexp(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                           hipStream_t s) {
  TX_ALL_DTYPES(LsePolicy)
  return launch<LsePolicy<uint8_t>>(p, x, out, c, ws, wsb, s);
}

}  // namespace red
}  // namespace tx
