// btc_gemv: argument checks and engine selection for the decode-time product.
#include "btc_internal.h"

namespace btc {
btc_status gemv_generic(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                        const float* alpha, const float* mu, const void* x, int batch, void* y, int y_is_f32);
}

extern "C" {

btc_status btc_gemv(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* x, int32_t batch, void* y, btc_dtype y_dtype,
                    void* workspace, size_t workspace_bytes) {
  using namespace btc;
  (void)workspace;
  (void)workspace_bytes;
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (!packed || !codebook || !alpha || !mu || !x || !y) return BTC_ERR_NULL;
  if (batch < 1 || batch > 16) return BTC_ERR_UNSUPPORTED;
  if (y_dtype != BTC_F16 && y_dtype != BTC_F32) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(packed) || !aligned16(codebook) || !aligned16(alpha) || !aligned16(mu) || !aligned16(x) ||
      !aligned16(y))
    return BTC_ERR_ALIGN;
  return gemv_generic((hipStream_t)stream, dims_of(*s), packed, codebook, alpha, mu, x, batch, y,
                      y_dtype == BTC_F32);
}

}  // extern "C"
