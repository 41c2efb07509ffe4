// btc_gemv: argument checks and engine selection for the decode-time product.
#include "btc_internal.h"

// Rough duration in microseconds of one decode pass over the matrix for a single activation
// row (a fixed chain of round trips plus streaming time; fitted to measurements on 7B-shaped
// layers).  Compared with the tiled contraction kernel's own estimate to decide whether a
// batch is served by one pass per row or by one pass of that kernel for all rows.
static double row_pass_us(const btc::Dims& d) { return 3.5 + 1.8e-6 * (double)d.out * d.wpr * 4; }

extern "C" {

btc_status btc_gemv(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* x, int32_t batch, void* y, btc_dtype y_dtype,
                    void* workspace, size_t workspace_bytes) {
  using namespace btc;
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (!packed || !codebook || !alpha || !mu || !x || !y) return BTC_ERR_NULL;
  if (batch < 1 || batch > 16) return BTC_ERR_UNSUPPORTED;
  if (y_dtype != BTC_F16 && y_dtype != BTC_F32) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(packed) || !aligned16(codebook) || !aligned16(alpha) || !aligned16(mu) || !aligned16(x) ||
      !aligned16(y))
    return BTC_ERR_ALIGN;
  hipStream_t q = (hipStream_t)stream;
  const Dims d = dims_of(*s);
  const int y_is_f32 = y_dtype == BTC_F32;
  const size_t ysz = y_is_f32 ? 4 : 2;
  // Several activation rows on a supported setting: one pass of the matrix-core engine serves them all
  // (unless the matrix is so small that a pass per row is still quicker).  A single row goes there
  // too when the matrix is large and so wide that the table engine cannot use its streaming kernel
  // (measured on 8192 x 28672: 22.7 against 29.9 us at 9 index bits, 23.2 against 38.8 us at 10).
  // One row, 9 or 10 index bits, a wide matrix with few enough rows: the single-kernel variant of the
  // matrix-core engine (measured on 4096 x 11008 at 9 bits: 8.6 us against 11.4 for the table engine; at 7 or
  // 8 bits, or with many rows, the other engines stay ahead).
  if (batch == 1 && d.b >= 9 && d.nchunks >= 1024 && d.out <= 6144 && gemv_mfma_one_covers(d))
    return gemv_mfma_one(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
  bool use_mfma = false;
  if (gemv_mfma_covers(d, batch)) {
    const long long bytes = (long long)d.out * d.wpr * 4;
    if (batch == 1)   // also every large matrix with 10-bit indices, where the table engine's 128 KB table
                      // allows one workgroup per compute unit only (28672 x 8192: 25.8 against 29.6 us)
      use_mfma = (d.b >= 9 && d.nchunks >= 2048 && bytes >= (16LL << 20)) || (d.b == 10 && bytes >= (8LL << 20));
    else use_mfma = batch * row_pass_us(d) > gemv_mfma_estimate_us(d, batch);
  }
  if (use_mfma) {
    const size_t off = gemv_table_region_bytes(d);
    const size_t need = gemv_mfma_workspace_bytes(d, batch);
    if (!workspace || workspace_bytes < off + need) return BTC_ERR_WORKSPACE;
    if (!aligned16(workspace)) return BTC_ERR_ALIGN;
    return gemv_mfma(q, d, packed, codebook, alpha, mu, x, /*is_bf16=*/0, batch, y, (int)y_dtype, (char*)workspace + off);
  }
  // Several activation rows: decoding the indices is the cost, and the matrix cores take up to 32
  // rows for the price of one, so the call goes to the tiled contraction kernel (each index is
  // decoded once for the whole batch) instead of one decode pass per row.
  if (batch > 1 && gemm_tiled_covers(d, batch) && batch * row_pass_us(d) > gemm_tiled_estimate_us(d, batch)) {
    // A k-split call parks partial sums in the workspace (after the table engine's slots of this
    // shape) and zeroes them again in its second pass, so that one zero-filled workspace serves
    // any sequence of calls, whatever their shapes and batch sizes.
    const size_t off = gemv_table_region_bytes(d);
    const size_t need = gemm_tiled_workspace_bytes(d, batch);
    if (need > 0) {
      if (!workspace || workspace_bytes < off + need) return BTC_ERR_WORKSPACE;
      if (!aligned16(workspace)) return BTC_ERR_ALIGN;
    }
    return gemm_tiled(q, d, packed, codebook, alpha, mu, x, /*is_bf16=*/0, batch, y, (int)y_dtype,
                      need > 0 ? (char*)workspace + off : nullptr, need, /*clear_workspace=*/1);
  }
  // Small matrices are bound by the chain of memory round trips: the register-resident engine has the
  // shortest one.  Larger ones are bound by LDS and ALU throughput, where the table engine is lighter
  // Measured crossover: 4096 x 4096 (1.5-1.9 MB) is faster expanded; at 5120 x 5120 (2.3-2.6 MB) the two
  // are within 0.5 us of each other -- expansion ahead on clustered (Zipf) indices, whose repeated table
  // reads LDS serves as broadcasts, the table engine ahead on uniform ones; from 4 MB on the table engine.
  const bool small = (long long)d.out * d.wpr * 4 < (3LL << 20) || !lut_engine_covers(d);
  if (small && expand_engine_covers(d)) {
    for (int m = 0; m < batch; ++m) {
      st = gemv_expand(q, d, packed, codebook, alpha, mu, (const char*)x + (size_t)m * d.in * 2,
                       (char*)y + (size_t)m * d.out * ysz, y_is_f32);
      if (st != BTC_OK) return st;
    }
    return BTC_OK;
  }
  if (!lut_engine_covers(d)) return gemv_generic(q, d, packed, codebook, alpha, mu, x, batch, y, y_is_f32);

  if (!workspace || workspace_bytes < btc_workspace_bytes(s, batch, 0)) return BTC_ERR_WORKSPACE;
  if (!aligned16(workspace)) return BTC_ERR_ALIGN;
  // One pass of the table engine per activation row; the passes share the
  // workspace, which is safe because they are ordered on the stream.
  for (int m = 0; m < batch; ++m) {
    st = gemv_lut(q, d, packed, codebook, alpha, mu, (const char*)x + (size_t)m * d.in * 2,
                  (char*)y + (size_t)m * d.out * ysz, y_is_f32, workspace);
    if (st != BTC_OK) return st;
  }
  return BTC_OK;
}

}  // extern "C"
