// The layer on quantised activations (section "Activation Quantization on sub-bit LLMs": W0.8A8, W0.8A4;
// appendix hyper-parameters: min-max quantisation, one scale per channel -- here one (offset, step) pair
// per activation row, since a scale that varied along the contraction index could not leave the integer sum):
//
//   btc_quantize_rows    q[m][k] = round((x[m][k] - lo[m]) / step[m]),  lo = row minimum,
//                        step = (row maximum - lo) / (2^bits - 1);  x ~ lo + step * q
//   btc_weight_rowsums   wsum[i] = sum_k W_hat[i][k]                      (once per layer)
//   btc_gemm_aq          y[m][i] = sum_k W_hat[i][k] (lo[m] + step[m] q[m][k])
//                                = step[m] * (alpha_i * sum_k B_hat[i][k] q[m][k] + mu_i * sum_k q[m][k]) + lo[m] * wsum[i]
//
// The integer sums are exact: the codes (0 .. 255) are exact in fp16 and bf16, products with +-1 and their
// fp32 sums stay below 2^24 for rows of up to 65793 weights, so the contraction is handed to the kernels
// of btc_gemv / btc_gemm with the codes as 16-bit operands, and an epilogue applies step, lo and wsum.
// Calls with enough rows to fill the chip go to the integer matrix cores instead (btc_gemm_wide_i8.hip).
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <algorithm>

#include "btc_internal.h"

namespace btc {
namespace aq {

constexpr int kThreads = 256;
constexpr int kMaxIn = 65536;           // integer row sums exact in fp32

__device__ __forceinline__ float widen16(uint16_t h, int is_bf16) {
  if (is_bf16) return __builtin_bit_cast(float, (uint32_t)h << 16);
  return __half2float(__builtin_bit_cast(__half, h));
}

// One workgroup per activation row, eight elements per load when the row allows it (n % 8 == 0; rows are
// then 16-byte aligned).  The decision arithmetic is fp32, one IEEE operation per step, in this order:
// t = x - lo;  r = t / step;  q = round-to-nearest-even(r) clamped to the grid.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void quantize_rows_kernel(const uint16_t* __restrict__ X, int is_bf16, int n,
                                                                 int bits, uint8_t* __restrict__ Q,
                                                                 float* __restrict__ lo, float* __restrict__ step,
                                                                 float* __restrict__ qsum) {
  __shared__ float red_min[kThreads / 64], red_max[kThreads / 64], red_sum[kThreads / 64];
  const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint16_t* x = X + (size_t)m * n;
  float mn = widen16(x[0], is_bf16), mx = mn;
  if (VEC) {
    for (int k = tid; k < n / 8; k += kThreads) {
      const uint4 v = ((const uint4*)x)[k];
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float f = widen16((uint16_t)(w[e >> 1] >> (16 * (e & 1))), is_bf16);
        mn = fminf(mn, f);
        mx = fmaxf(mx, f);
      }
    }
  } else {
    for (int k = tid; k < n; k += kThreads) {
      const float v = widen16(x[k], is_bf16);
      mn = fminf(mn, v);
      mx = fmaxf(mx, v);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, o, 64));
    mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  }
  if (lane == 0) {
    red_min[wave] = mn;
    red_max[wave] = mx;
  }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) {
    mn = fminf(mn, red_min[w]);
    mx = fmaxf(mx, red_max[w]);
  }
  const float levels = (float)((1 << bits) - 1);
  const float range = mx - mn;
  const float st = range > 0.0f ? range / levels : 1.0f;
  float sum = 0.f;                                       // integers: exact in any order
  // The decision is rint(t / step) with an IEEE division.  t * (1 / step) differs from the quotient by at most
  // a few 2^-24 of it, less than 1e-4 on a grid of 255 levels, so it rounds to the same integer unless it lies
  // within 1e-3 of a half: only those elements (about one in 500) pay for the division.
  const float inv = 1.0f / st;
  auto code = [&](uint16_t h) -> uint32_t {
    const float t = widen16(h, is_bf16) - mn;
    const float r0 = t * inv;
    float r = rintf(r0);
    if (fabsf(fabsf(r0 - r) - 0.5f) < 1e-3f) r = rintf(t / st);
    r = fminf(fmaxf(r, 0.0f), levels);
    sum += r;
    return (uint32_t)(int)r;
  };
  if (VEC) {
    for (int k = tid; k < n / 8; k += kThreads) {        // (a second read of the row: it is in the L2)
      const uint4 v = ((const uint4*)x)[k];
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      uint32_t o[2] = {0u, 0u};
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e >> 2] |= code((uint16_t)(w[e >> 1] >> (16 * (e & 1)))) << (8 * (e & 3));
      ((uint2*)(Q + (size_t)m * n))[k] = make_uint2(o[0], o[1]);
    }
  } else {
    for (int k = tid; k < n; k += kThreads) Q[(size_t)m * n + k] = (uint8_t)code(x[k]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
  if (lane == 0) red_sum[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) s += red_sum[w];
    lo[m] = mn;
    step[m] = st;
    if (qsum) qsum[m] = s;
  }
}

// codes -> the same integers as fp16 numbers (exact), the operand format of the contraction kernels
__global__ __launch_bounds__(kThreads) void widen_codes_kernel(const uint8_t* __restrict__ Q, size_t count,
                                                               uint16_t* __restrict__ Q16) {
  const size_t i = ((size_t)blockIdx.x * kThreads + threadIdx.x) * 4;
  if (i + 3 < count) {
    const uint32_t w = *(const uint32_t*)(Q + i);
    uint16_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = __builtin_bit_cast(uint16_t, __float2half_rn((float)((w >> (8 * e)) & 0xFFu)));
    *(uint2*)(Q16 + i) = make_uint2(o[0] | ((uint32_t)o[1] << 16), o[2] | ((uint32_t)o[3] << 16));
  } else {
    for (size_t j = i; j < count; ++j) Q16[j] = __builtin_bit_cast(uint16_t, __float2half_rn((float)Q[j]));
  }
}

// (a fill kernel rather than a memset node: callers may capture these calls in a graph)
__global__ __launch_bounds__(kThreads) void zero_kernel(uint4* __restrict__ p, size_t n16) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

__global__ __launch_bounds__(kThreads) void fill_ones_kernel(uint16_t* __restrict__ x, int n) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < n) x[i] = 0x3C00u;   // 1.0 in fp16
}

// Y[m][i] = step[m] * T[m][i] + lo[m] * wsum[i]
__global__ __launch_bounds__(kThreads) void aq_epilogue_kernel(const float* __restrict__ T, const float* __restrict__ lo,
                                                               const float* __restrict__ step,
                                                               const float* __restrict__ wsum, int M, int out,
                                                               void* __restrict__ Y, int y_dtype) {
  const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= (size_t)M * out) return;
  const int m = (int)(idx / out), i = (int)(idx - (size_t)m * out);
  const float r = step[m] * T[idx] + lo[m] * wsum[i];
  if (y_dtype == BTC_F32) ((float*)Y)[idx] = r;
  else if (y_dtype == BTC_BF16) ((__hip_bfloat16*)Y)[idx] = __float2bfloat16(r);
  else ((__half*)Y)[idx] = __float2half_rn(r);
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static btc_status zero_fill(hipStream_t q, void* p, size_t bytes) {
  const size_t n16 = (bytes + 15) / 16;                  // the regions are multiples of 256 bytes
  if (n16 == 0) return BTC_OK;
  zero_kernel<<<(unsigned)((n16 + kThreads - 1) / kThreads), kThreads, 0, q>>>((uint4*)p, n16);
  return launch_status();
}

}  // namespace aq
}  // namespace btc

extern "C" {

btc_status btc_quantize_rows(void* stream, const void* X, btc_dtype x_dtype, int32_t M, int32_t n, int32_t bits,
                             uint8_t* Q, float* lo, float* step, float* qsum) {
  using namespace btc;
  if (!X || !Q || !lo || !step) return BTC_ERR_NULL;
  if (M <= 0 || n <= 0) return BTC_ERR_SHAPE;
  if ((bits != 8 && bits != 4) || (x_dtype != BTC_F16 && x_dtype != BTC_BF16) || n > aq::kMaxIn) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(X) || !aligned16(Q) || !aligned16(lo) || !aligned16(step) || (qsum && !aligned16(qsum))) return BTC_ERR_ALIGN;
  if (n % 8 == 0)
    aq::quantize_rows_kernel<true><<<M, aq::kThreads, 0, (hipStream_t)stream>>>((const uint16_t*)X, x_dtype == BTC_BF16, n,
                                                                                 bits, Q, lo, step, qsum);
  else
    aq::quantize_rows_kernel<false><<<M, aq::kThreads, 0, (hipStream_t)stream>>>((const uint16_t*)X, x_dtype == BTC_BF16, n,
                                                                                  bits, Q, lo, step, qsum);
  return launch_status();
}

size_t btc_aq_workspace_bytes(const btc_shape* s, int32_t M) {
  using namespace btc;
  if (!s || M <= 0) return 0;
  const int rows = M < 1 ? 1 : M;
  const size_t inner = M <= 16 ? btc_workspace_bytes(s, rows, 0) : btc_workspace_bytes(s, rows, 1);
  // 16-bit copy of the codes (or the row of ones of btc_weight_rowsums), the fp32 result of the
  // contraction, then the contraction's own workspace
  size_t need = aq::align256((size_t)rows * s->in * 2) + aq::align256((size_t)rows * s->out * 4) + aq::align256(inner);
  // many rows: the sign matrix as int8 and the sums of the code rows, for the integer matrix cores
  const Dims d = dims_of(*s);
  if (gemm_wide_i8_covers(d, M)) need = std::max(need, aq::align256(gemm_wide_i8_workspace_bytes(d, M)));
  return need;
}

btc_status btc_weight_rowsums(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                              const float* alpha, const float* mu, float* wsum, void* workspace, size_t workspace_bytes) {
  using namespace btc;
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (!packed || !codebook || !alpha || !mu || !wsum || !workspace) return BTC_ERR_NULL;
  if (!aligned16(wsum) || !aligned16(workspace)) return BTC_ERR_ALIGN;
  if (workspace_bytes < btc_aq_workspace_bytes(s, 1)) return BTC_ERR_WORKSPACE;
  // W_hat . 1: the decode product on a row of ones (exact integers inside, one rounding per term outside)
  uint16_t* ones = (uint16_t*)workspace;
  char* inner = (char*)workspace + aq::align256((size_t)s->in * 2) + aq::align256((size_t)s->out * 4);
  const size_t inner_bytes = btc_workspace_bytes(s, 1, 0);
  hipStream_t q = (hipStream_t)stream;
  if (gemv_auto_uses_workspace(dims_of(*s), 1)) {
    st = aq::zero_fill(q, inner, inner_bytes);
    if (st != BTC_OK) return st;
  }
  aq::fill_ones_kernel<<<(s->in + aq::kThreads - 1) / aq::kThreads, aq::kThreads, 0, q>>>(ones, s->in);
  st = launch_status();
  if (st != BTC_OK) return st;
  return btc_gemv(stream, s, packed, codebook, alpha, mu, ones, 1, wsum, BTC_F32, inner, inner_bytes);
}

btc_status btc_gemm_aq(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                       const float* alpha, const float* mu, const float* wsum, const uint8_t* Q, const float* lo,
                       const float* step, int32_t M, void* Y, btc_dtype y_dtype, void* workspace,
                       size_t workspace_bytes) {
  using namespace btc;
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (!packed || !codebook || !alpha || !mu || !wsum || !Q || !lo || !step || !Y || !workspace) return BTC_ERR_NULL;
  if (M <= 0) return BTC_ERR_SHAPE;
  if (s->in > aq::kMaxIn) return BTC_ERR_UNSUPPORTED;
  if (y_dtype != BTC_F32 && y_dtype != BTC_F16 && y_dtype != BTC_BF16) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(wsum) || !aligned16(Q) || !aligned16(lo) || !aligned16(step) || !aligned16(Y) || !aligned16(workspace))
    return BTC_ERR_ALIGN;
  if (workspace_bytes < btc_aq_workspace_bytes(s, M)) return BTC_ERR_WORKSPACE;
  hipStream_t q = (hipStream_t)stream;
  {
    const Dims d = dims_of(*s);
    if (gemm_wide_i8_covers(d, M))   // enough rows to fill the chip: int8 operands on the integer matrix cores
      return gemm_wide_i8(q, d, packed, codebook, alpha, mu, wsum, Q, lo, step, M, Y, (int)y_dtype, workspace,
                          workspace_bytes);
  }
  uint16_t* Q16 = (uint16_t*)workspace;
  float* T = (float*)((char*)workspace + aq::align256((size_t)M * s->in * 2));
  char* inner = (char*)T + aq::align256((size_t)M * s->out * 4);
  const size_t inner_bytes = M <= 16 ? btc_workspace_bytes(s, M, 0) : btc_workspace_bytes(s, M, 1);
  const size_t count = (size_t)M * s->in;
  aq::widen_codes_kernel<<<(unsigned)((count / 4 + aq::kThreads) / aq::kThreads), aq::kThreads, 0, q>>>(Q, count, Q16);
  st = launch_status();
  if (st != BTC_OK) return st;
  if (M <= 16) {
    // the decode engines that park partial sums want their workspace zero-filled and hand it back that way
    if (gemv_auto_uses_workspace(dims_of(*s), M)) {
      st = aq::zero_fill(q, inner, inner_bytes);
      if (st != BTC_OK) return st;
    }
    st = btc_gemv(stream, s, packed, codebook, alpha, mu, Q16, M, T, BTC_F32, inner, inner_bytes);
  } else {
    st = btc_gemm(stream, s, packed, codebook, alpha, mu, Q16, BTC_F16, M, T, BTC_F32, inner, inner_bytes);
  }
  if (st != BTC_OK) return st;
  const size_t total = (size_t)M * s->out;
  aq::aq_epilogue_kernel<<<(unsigned)((total + aq::kThreads - 1) / aq::kThreads), aq::kThreads, 0, q>>>(
      T, lo, step, wsum, M, s->out, Y, (int)y_dtype);
  return launch_status();
}

}  // extern "C"
