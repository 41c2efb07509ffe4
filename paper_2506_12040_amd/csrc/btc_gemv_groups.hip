// Decode-time product for the storage variant with several (alpha, mu) pairs per weight row (Table "Study
// of Number of Split Points"; appendix hyper-parameters: 2 split points by default, 3 for higher accuracy):
//   W_hat[i][k] = alpha[i][g] * B_hat[i][k] + mu[i][g],   g = group[i][k] in [0, G),  G <= 4
//   y[i] = sum_g ( alpha[i][g] * sum_{k in g} B_hat[i][k] x[k]  +  mu[i][g] * sum_{k in g} x[k] )
// The partition is an explicit map of 2 bits per weight (bits [2k, 2k+2) of row i's map, LSB-first like the
// index stream, ceil(2 in / 32) words per row): three times the bytes of a 0.8-bit index stream, which is
// why this is a variant and not the format of the tuned engines.  One wave per output row at a time, lane
// l takes chunks l, l + 64, ..; per weight the sign is applied and the value added to its group's two
// sums (branch-free: one fused multiply-add per group with a 0/1 factor); fp32 sums, fixed order.
#include <hip/hip_fp16.h>

#include <algorithm>

#include "btc_internal.h"

namespace btc {
namespace groups {

constexpr int kWaves = 16;
constexpr int kMaxIn = 32768;           // activation row in LDS: 64 KB
constexpr int kCodebookLds = 8192;      // codebook entries held in LDS (32 KB)

__device__ __forceinline__ float wave_sum(float a) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
  return a;
}

template <int G, bool CB_LDS>
__global__ __launch_bounds__(kWaves * 64) void gemv_groups_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                                  const uint32_t* __restrict__ codebook,
                                                                  const float* __restrict__ alpha,
                                                                  const float* __restrict__ mu,
                                                                  const uint32_t* __restrict__ gmap,
                                                                  const uint16_t* __restrict__ x, void* __restrict__ y,
                                                                  int y_is_f32) {
  extern __shared__ __align__(16) unsigned char smem[];
  __half* xs = (__half*)smem;                            // [in]
  uint32_t* cb = (uint32_t*)(smem + (((size_t)d.in * 2 + 15) & ~(size_t)15));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int k = tid; k < d.in; k += kWaves * 64) xs[k] = __builtin_bit_cast(__half, x[k]);
  if (CB_LDS)
    for (int k = tid; k < (1 << d.b); k += kWaves * 64) cb[k] = codebook[k];
  __syncthreads();
  const uint32_t mask = (1u << d.b) - 1u;
  const int gwpr = (2 * d.in + 31) >> 5;
  for (int i = blockIdx.x * kWaves + wave; i < d.out; i += gridDim.x * kWaves) {
    const uint32_t* row = packed + (size_t)i * d.wpr;
    const uint32_t* grow = gmap + (size_t)i * gwpr;
    float acc[G], sx[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = sx[g] = 0.f;
    for (int j = lane; j < d.nchunks; j += 64) {
      const uint32_t p = (uint32_t)j * (uint32_t)d.b;
      const uint32_t w = p >> 5, sh = p & 31u;
      const uint32_t lo = row[w];
      const uint32_t hi = (sh + d.b > 32u) ? row[w + 1] : 0u;   // inside the row whenever the field crosses
      const uint32_t code = __builtin_amdgcn_alignbit(hi, lo, sh) & mask;
      const uint32_t pat = CB_LDS ? cb[code] : codebook[code];
      const int k0 = j * d.v;
      const int len = min(d.v, d.in - k0);
      // the 2 * len <= 64 map bits of the chunk: three words cover them whatever the alignment
      const int gw = (2 * k0) >> 5;
      const uint32_t gs = (uint32_t)(2 * k0) & 31u;
      const uint32_t g0 = grow[gw];
      const uint32_t g1 = gw + 1 < gwpr ? grow[gw + 1] : 0u;
      const uint32_t g2 = gw + 2 < gwpr ? grow[gw + 2] : 0u;
      const uint32_t mlo = __builtin_amdgcn_alignbit(g1, g0, gs), mhi = __builtin_amdgcn_alignbit(g2, g1, gs);
      for (int t = 0; t < len; ++t) {
        const float xv = __half2float(xs[k0 + t]);
        const float sv = ((pat >> t) & 1u) ? xv : -xv;
        const uint32_t gi = ((t < 16 ? mlo : mhi) >> (2 * (t & 15))) & 3u;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float on = gi == (uint32_t)g ? 1.0f : 0.0f;
          acc[g] = fmaf(on, sv, acc[g]);
          sx[g] = fmaf(on, xv, sx[g]);
        }
      }
    }
    float r = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float a = wave_sum(acc[g]), sxx = wave_sum(sx[g]);
      r += alpha[(size_t)i * G + g] * a + mu[(size_t)i * G + g] * sxx;
    }
    if (lane == 0) {
      if (y_is_f32) ((float*)y)[i] = r;
      else ((__half*)y)[i] = __float2half_rn(r);
    }
  }
}

template <int G>
static btc_status launch(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                         const float* alpha, const float* mu, const uint32_t* gmap, const void* x, void* y, int y_is_f32) {
  const bool cb_lds = (1 << d.b) <= kCodebookLds;
  const size_t lds = (((size_t)d.in * 2 + 15) & ~(size_t)15) + (cb_lds ? (size_t)4 << d.b : 0);
  const int grid = std::min(512, (d.out + kWaves - 1) / kWaves);
  static bool attr_set = false;  // one-time kernel attributes, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemv_groups_kernel<G, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess ||
        hipFuncSetAttribute((const void*)gemv_groups_kernel<G, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  if (cb_lds)
    gemv_groups_kernel<G, true><<<grid, kWaves * 64, lds, q>>>(d, packed, codebook, alpha, mu, gmap, (const uint16_t*)x, y, y_is_f32);
  else
    gemv_groups_kernel<G, false><<<grid, kWaves * 64, lds, q>>>(d, packed, codebook, alpha, mu, gmap, (const uint16_t*)x, y, y_is_f32);
  return launch_status();
}

}  // namespace groups
}  // namespace btc

extern "C" btc_status btc_gemv_groups(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                                      const float* alpha, const float* mu, const uint32_t* group_map, int32_t ngroups,
                                      const void* x, void* y, btc_dtype y_dtype) {
  using namespace btc;
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (!packed || !codebook || !alpha || !mu || !group_map || !x || !y) return BTC_ERR_NULL;
  if (ngroups < 1 || ngroups > 4 || s->in > groups::kMaxIn) return BTC_ERR_UNSUPPORTED;
  if (y_dtype != BTC_F16 && y_dtype != BTC_F32) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(packed) || !aligned16(codebook) || !aligned16(alpha) || !aligned16(mu) || !aligned16(group_map) ||
      !aligned16(x) || !aligned16(y))
    return BTC_ERR_ALIGN;
  const Dims d = dims_of(*s);
  hipStream_t q = (hipStream_t)stream;
  const int f32 = y_dtype == BTC_F32;
  switch (ngroups) {
    case 1: return groups::launch<1>(q, d, packed, codebook, alpha, mu, group_map, x, y, f32);
    case 2: return groups::launch<2>(q, d, packed, codebook, alpha, mu, group_map, x, y, f32);
    case 3: return groups::launch<3>(q, d, packed, codebook, alpha, mu, group_map, x, y, f32);
    default: return groups::launch<4>(q, d, packed, codebook, alpha, mu, group_map, x, y, f32);
  }
}
