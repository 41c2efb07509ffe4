// Generic decode-time product: any chunk length v <= 32, any index width
// b <= 16, batch 1..16, reading the canonical per-row bit stream.
//
// One 64-lane wave owns one output row.  Lane l walks chunks l, l+64, ...:
// it extracts the chunk's index from the stream, fetches the sign pattern
// (codebook in LDS when it fits) and applies the signs to the chunk's
// activations on the vector ALU, i.e. it evaluates the blockwise dot product
// <x_j, C[I_rj]> of appendix "Binary Codebook LUT-GEMM" directly, without
// tables.  Row sums are reduced across the wave by shuffles; the epilogue
// applies y = alpha * acc + mu * sum(x) (dequantisation step of Algorithm
// "Binary Transformation and Compression").  This kernel is the fallback for
// settings the tuned engines do not cover.
#include <hip/hip_fp16.h>

#include "btc_internal.h"

namespace btc {

constexpr int kGenericCodebookLdsEntries = 8192;  // 32 KB

__device__ __forceinline__ float wave_sum(float a) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
  return a;
}

template <int BT, bool CB_LDS>
__global__ __launch_bounds__(256) void gemv_generic_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                           const uint32_t* __restrict__ codebook,
                                                           const float* __restrict__ alpha,
                                                           const float* __restrict__ mu,
                                                           const __half* __restrict__ x, int batch,
                                                           void* __restrict__ y, int y_is_f32) {
  __shared__ uint32_t cb_lds[CB_LDS ? kGenericCodebookLdsEntries : 1];
  const int ncode = 1 << d.b;
  if (CB_LDS) {
    for (int k = threadIdx.x; k < ncode; k += blockDim.x) cb_lds[k] = codebook[k];
    __syncthreads();
  }
  const uint32_t* cb = CB_LDS ? cb_lds : codebook;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int waves_per_block = blockDim.x >> 6;

  for (int i = blockIdx.x * waves_per_block + wave; i < d.out; i += gridDim.x * waves_per_block) {
    const uint32_t* row = packed + (long long)i * d.wpr;
    float acc[BT], sx[BT];
#pragma unroll
    for (int m = 0; m < BT; ++m) acc[m] = sx[m] = 0.f;
    for (int j = lane; j < d.nchunks; j += 64) {
      const uint32_t pat = cb[field_at(row, d.wpr, j * d.b, d.b)];
      const int k0 = j * d.v;
      const int len = min(d.v, d.in - k0);
      for (int t = 0; t < len; ++t) {
        const bool plus = (pat >> t) & 1u;
#pragma unroll
        for (int m = 0; m < BT; ++m) {
          if (m < batch) {
            const float xv = __half2float(x[(long long)m * d.in + k0 + t]);
            acc[m] += plus ? xv : -xv;
            sx[m] += xv;
          }
        }
      }
    }
    const float a = alpha[i], mm = mu[i];
#pragma unroll
    for (int m = 0; m < BT; ++m) {
      if (m < batch) {
        const float r = a * wave_sum(acc[m]) + mm * wave_sum(sx[m]);
        if (lane == 0) {
          if (y_is_f32) ((float*)y)[(long long)m * d.out + i] = r;
          else ((__half*)y)[(long long)m * d.out + i] = __float2half_rn(r);
        }
      }
    }
  }
}

template <int BT>
static void launch_generic(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                           const float* alpha, const float* mu, const void* x, int batch, void* y, int y_is_f32) {
  const int blocks = (d.out + 3) / 4;
  if ((1 << d.b) <= kGenericCodebookLdsEntries)
    gemv_generic_kernel<BT, true><<<blocks, 256, 0, q>>>(d, packed, codebook, alpha, mu, (const __half*)x, batch, y, y_is_f32);
  else
    gemv_generic_kernel<BT, false><<<blocks, 256, 0, q>>>(d, packed, codebook, alpha, mu, (const __half*)x, batch, y, y_is_f32);
}

btc_status gemv_generic(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                        const float* alpha, const float* mu, const void* x, int batch, void* y, int y_is_f32) {
  if (batch == 1) launch_generic<1>(q, d, packed, codebook, alpha, mu, x, batch, y, y_is_f32);
  else if (batch <= 4) launch_generic<4>(q, d, packed, codebook, alpha, mu, x, batch, y, y_is_f32);
  else launch_generic<16>(q, d, packed, codebook, alpha, mu, x, batch, y, y_is_f32);
  return launch_status();
}

}  // namespace btc
