// Instantiates the prod / amax / argmax reduction policies.
#include "reduce_impl.h"

namespace tx {
namespace red {

#define TX_ALL_DTYPES(POLICY)                                                          \
  switch (x->dtype) {                                                                  \
    case TX_F32: return launch<POLICY<float>>(p, x, out, c, ws, wsb, s);                \
    case TX_BF16: return launch<POLICY<bf16>>(p, x, out, c, ws, wsb, s);                \
    case TX_F16: return launch<POLICY<f16>>(p, x, out, c, ws, wsb, s);                  \
    case TX_I64: return launch<POLICY<int64_t>>(p, x, out, c, ws, wsb, s);              \
    case TX_I32: return launch<POLICY<int32_t>>(p, x, out, c, ws, wsb, s);              \
    default: break;                                                                    \
  }

tx_status launch_prod(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                      hipStream_t s) {
  TX_ALL_DTYPES(ProdPolicy)
  return launch<ProdPolicy<uint8_t>>(p, x, out, c, ws, wsb, s);
}

tx_status launch_amax(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                      hipStream_t s) {
  TX_ALL_DTYPES(AmaxPolicy)
  return launch<AmaxPolicy<uint8_t>>(p, x, out, c, ws, wsb, s);
}

tx_status launch_argmax(const Plan& p, const tx_tensor* x, const tx_tensor* out, double c, void* ws, size_t wsb,
                        hipStream_t s) {
  TX_ALL_DTYPES(ArgmaxPolicy)
  return fail(TX_ERR_DTYPE, "argmax does not take bool");
}

}  // namespace red
}  // namespace tx
