// btc_gemm: argument checks, the fp32 row sums of X, and kernel selection for
// the prefill product  Y[M][out] = X[M][in] . W_hat^T.
//
// The affine part of the dequantisation (Algorithm "Binary Transformation and
// Compression": W_hat = alpha * B_hat + mu) is applied after the contraction:
//     Y[m][i] = alpha_i * sum_k X[m][k] s[i][k]  +  mu_i * sum_k X[m][k],
// so the kernels contract X with the exact +-1 patterns and need sum_k X[m][k].
#include <hip/hip_fp16.h>

#include "btc_internal.h"

namespace btc {

__device__ __forceinline__ float load_as_float(const uint16_t* p, bool bf16) {
  const uint16_t h = *p;
  if (bf16) return __uint_as_float((uint32_t)h << 16);
  return __half2float(__ushort_as_half(h));
}

// rowsum[m] = sum_k X[m][k] in fp32, one wave per row, fixed order: lane l adds
// elements 8l..8l+7 of every block of 512 (16-byte loads), then the lanes are
// added by a butterfly.  Rows whose length is not a multiple of 8 take the
// element-wise path.
__global__ __launch_bounds__(256) void rowsum_kernel(const uint16_t* __restrict__ X, int M, int in, int is_bf16,
                                                     float* __restrict__ rowsum) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= M) return;
  const uint16_t* row = X + (long long)m * in;
  float s = 0.f;
  if ((in & 7) == 0) {
    for (int k = lane * 8; k < in; k += 512) {
      const uint4 v = *(const uint4*)(row + k);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (is_bf16) {
          s += __uint_as_float(w[i] << 16);
          s += __uint_as_float(w[i] & 0xFFFF0000u);
        } else {
          s += __half2float(__ushort_as_half((uint16_t)(w[i] & 0xFFFFu)));
          s += __half2float(__ushort_as_half((uint16_t)(w[i] >> 16)));
        }
      }
    }
  } else {
    for (int k = lane; k < in; k += 64) s += load_as_float(row + k, is_bf16 != 0);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (lane == 0) rowsum[m] = s;
}

}  // namespace btc

extern "C" {

btc_status btc_gemm(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* X, btc_dtype x_dtype, int32_t M, void* Y,
                    btc_dtype y_dtype, void* workspace, size_t workspace_bytes) {
  using namespace btc;
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (!packed || !codebook || !alpha || !mu || !X || !Y) return BTC_ERR_NULL;
  if (M <= 0) return BTC_ERR_SHAPE;
  if (x_dtype != BTC_BF16 && x_dtype != BTC_F16) return BTC_ERR_UNSUPPORTED;
  if (y_dtype != BTC_F32 && y_dtype != BTC_BF16 && y_dtype != BTC_F16) return BTC_ERR_UNSUPPORTED;
  if (!workspace || workspace_bytes < btc_workspace_bytes(s, M, 1)) return BTC_ERR_WORKSPACE;
  if (!aligned16(packed) || !aligned16(codebook) || !aligned16(alpha) || !aligned16(mu) || !aligned16(X) ||
      !aligned16(Y) || !aligned16(workspace))
    return BTC_ERR_ALIGN;
  hipStream_t q = (hipStream_t)stream;
  const Dims d = dims_of(*s);
  float* rowsum = (float*)((char*)workspace + 16);
  const int is_bf16 = x_dtype == BTC_BF16;
  // 17..64 activation rows: the same operand scheme with two or four blocks of activation rows
  // per table read, one pass over the index stream.
  if (gemm_rows_covers(d, M) &&
      gemm_rows_estimate_us(d, M) < (gemm_tiled_covers(d, M) ? gemm_tiled_estimate_us(d, M) : 1e30))
    return gemm_rows(q, d, packed, codebook, alpha, mu, X, is_bf16, M, Y, (int)y_dtype, workspace);
  // 65..128 rows on a large matrix (6 MB of indices or more): two passes of that kernel (64 rows, then
  // the rest) still beat a 256-row tile that is half empty (8192 x 28672, M = 96: 77 against 118 us); the
  // estimates decide.
  if (M > 64 && M <= 128 && (long long)d.out * d.wpr * 4 >= (6LL << 20) && gemm_rows_covers(d, 64) &&
      gemm_tiled_covers(d, M)) {
    const int rest = M - 64;
    const double est = gemm_rows_estimate_us(d, 64) +
                       (rest >= 17 ? gemm_rows_estimate_us(d, rest) : gemv_mfma_estimate_us(d, rest));
    if (1.1 * est < gemm_tiled_estimate_us(d, M)) {
      const size_t ysz = y_dtype == BTC_F32 ? 4 : 2;
      st = gemm_rows(q, d, packed, codebook, alpha, mu, X, is_bf16, 64, Y, (int)y_dtype, workspace);
      if (st != BTC_OK) return st;
      const void* X2 = (const char*)X + (size_t)64 * d.in * 2;
      void* Y2 = (char*)Y + (size_t)64 * d.out * ysz;
      if (rest >= 17) return gemm_rows(q, d, packed, codebook, alpha, mu, X2, is_bf16, rest, Y2, (int)y_dtype, workspace);
      return gemv_mfma(q, d, packed, codebook, alpha, mu, X2, is_bf16, rest, Y2, (int)y_dtype, workspace);
    }
  }
  // Few activation rows: decoding dominates, and the decode engine of btc_gemv (table entries
  // that are matrix-core operands, 16 rows per pass) is several times quicker than a 256-row tile
  // that is mostly empty.  Up to 64 rows are served in blocks of 16.
  if (M <= 64 && gemv_mfma_covers(d, M < 16 ? M : 16) &&
      ((M + 15) / 16) * gemv_mfma_estimate_us(d, M < 16 ? M : 16) <
          (gemm_tiled_covers(d, M) ? gemm_tiled_estimate_us(d, M) : 1e30)) {
    const size_t xsz = 2, ysz = y_dtype == BTC_F32 ? 4 : 2;
    for (int m0 = 0; m0 < M; m0 += 16) {
      const int rows = M - m0 < 16 ? M - m0 : 16;
      st = gemv_mfma(q, d, packed, codebook, alpha, mu, (const char*)X + (size_t)m0 * d.in * xsz, is_bf16, rows,
                     (char*)Y + (size_t)m0 * d.out * ysz, (int)y_dtype, workspace);
      if (st != BTC_OK) return st;
    }
    return BTC_OK;
  }
  // many rows and enough output tiles to fill the chip: expand the signs once, stream both operands (if the caller's workspace holds the bytes)
  if (gemm_wide_covers(d, M) && workspace && workspace_bytes >= gemm_wide_workspace_bytes(d, M))
    return gemm_wide(q, d, packed, codebook, alpha, mu, X, is_bf16, M, Y, (int)y_dtype, workspace, workspace_bytes);
  if (gemm_tiled_covers(d, M))   // adds the activation rows up itself
    return gemm_tiled(q, d, packed, codebook, alpha, mu, X, is_bf16, M, Y, (int)y_dtype, workspace, workspace_bytes,
                      /*clear_workspace=*/0);
  rowsum_kernel<<<(M + 3) / 4, 256, 0, q>>>((const uint16_t*)X, M, d.in, is_bf16, rowsum);
  return gemm_generic(q, d, packed, codebook, alpha, mu, X, is_bf16, M, Y, (int)y_dtype, rowsum);
}

}  // extern "C"
