// btc_transform: the online activation transform that precedes the layer at inference,
//     X <- X T,   T = D P,   D = diag(sigma), sigma_k = +-1,   P = P1 (x) P2
// (section "Learnable Transformation": transformation pair, Kronecker-factored P;
// "Integration into Transformer Architecture": Y = X W^T = (X T)(T^-1 W^T), the weights
// are compressed after T^-1 was folded in, the activations are transformed on the fly).
//
// A Kronecker-factored P never has to be formed: with a row of X reshaped to n1 x n2
// (channel i = i1 n2 + i2),  row . (P1 (x) P2)  reshaped the same way is  P1^T (X_m) P2.
// That is 2 n (n1 + n2) flop per row against 2 n^2 for the full matrix (144 against 5120
// multiply-adds per channel at n = 5120 = 64 x 80).
//
// Work split.  Output column j = j1 n2 + j2 depends on column j2 of P2 only, so a block of
// kCB columns j2 of ALL rows j1 is computed by one workgroup without help from any other:
//   stage 1:  Y1[i1][jj] = sum_i2 sigma x[i1 n2 + i2] P2[i2][j0 + jj]      (n1 x kCB values)
//   stage 2:  Z[j1][jj]  = sum_i1 P1[i1][j1] Y1[i1][jj]
// The workgroup keeps P1, its slice of P2 and the sign bits in LDS and walks over the rows of
// X dealt to it; a row is staged with its signs applied (a flip of the sign bit: exact).
// fp32 accumulation in ascending i2, then ascending i1: deterministic.  One activation row
// (decode) is n2 / kCB workgroups whose chain is: loads, stage 1, stage 2, store.
#include <hip/hip_fp16.h>

#include "btc_internal.h"

namespace btc {
namespace transform {

constexpr int kThreads = 256;
constexpr int kCB = 8;         // columns of P2 per workgroup
constexpr int kMaxN1 = 128;
constexpr int kMaxN2 = 256;

struct Layout {                // byte offsets into dynamic LDS
  int rs;                      // staged row stride in 16-bit elements (even; rs / 2 odd: rows start in different banks)
  int p1, p2, y1, sg, total;
};

static Layout layout_of(int n1, int n2) {
  Layout L;
  L.rs = 2 * (((n2 + 1) / 2) | 1);
  auto up16 = [](int b) { return (b + 15) & ~15; };
  L.p1 = up16(n1 * L.rs * 2);
  L.p2 = L.p1 + up16(n1 * n1 * 4);
  L.y1 = L.p2 + up16(n2 * kCB * 4);
  L.sg = L.y1 + up16(n1 * kCB * 4);
  L.total = L.sg + up16(((n1 * n2 + 31) / 32) * 4);
  return L;
}

template <bool BF16>
__device__ __forceinline__ float widen(uint32_t h) {
  if constexpr (BF16) return __uint_as_float(h << 16);
  else return __half2float(__ushort_as_half((uint16_t)h));
}

__device__ __forceinline__ void store_out(void* Y, size_t at, float v, int y_dtype) {
  if (y_dtype == BTC_F32) {
    ((float*)Y)[at] = v;
  } else if (y_dtype == BTC_F16) {
    ((__half*)Y)[at] = __float2half_rn(v);
  } else {                                   // bf16, round to nearest even (NaN stays NaN)
    const uint32_t u = __float_as_uint(v);
    const uint32_t r = (u & 0x7FFFFFFFu) > 0x7F800000u ? (u | 0x00400000u) : u + 0x7FFFu + ((u >> 16) & 1u);
    ((uint16_t*)Y)[at] = (uint16_t)(r >> 16);
  }
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void transform_kernel(const uint16_t* __restrict__ X, int M, int n1, int n2,
                                                            const uint32_t* __restrict__ sign_bits,
                                                            const float* __restrict__ P1,
                                                            const float* __restrict__ P2, void* __restrict__ Y,
                                                            int y_dtype, Layout L) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xs = (uint16_t*)smem;
  float* p1s = (float*)(smem + L.p1);
  float* p2s = (float*)(smem + L.p2);
  float* y1 = (float*)(smem + L.y1);
  uint32_t* sg = (uint32_t*)(smem + L.sg);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = n1 * n2;
  const int j0 = blockIdx.x * kCB;
  const int ncol = min(kCB, n2 - j0);

  // ---- once per workgroup: P1, columns j0 .. j0 + kCB - 1 of P2 (zero past the last column), sign words
  for (int t = tid; t < n1 * n1; t += kThreads) p1s[t] = P1[t];
  for (int t = tid; t < n2 * kCB; t += kThreads) {
    const int i2 = t / kCB, jj = t - i2 * kCB;
    p2s[t] = jj < ncol ? P2[(size_t)i2 * n2 + j0 + jj] : 0.f;
  }
  for (int t = tid; t < (n + 31) / 32; t += kThreads) sg[t] = sign_bits[t];

  const int items = n1 * (kCB / 2);          // an item: one row index and a pair of columns
  for (int m = blockIdx.y; m < M; m += gridDim.y) {
    __syncthreads();                         // sign words are there; the previous row's readers are done
    // ---- row m with its signs applied -> LDS, one wave per row i1 of the n1 x n2 view
    const uint16_t* xrow = X + (size_t)m * n;
    for (int i1 = wave; i1 < n1; i1 += kThreads / 64) {
      for (int i2 = lane; i2 < n2; i2 += 64) {
        const int k = i1 * n2 + i2;
        const uint32_t plus = (sg[k >> 5] >> (k & 31)) & 1u;
        xs[i1 * L.rs + i2] = (uint16_t)(xrow[k] ^ (plus ? 0u : 0x8000u));
      }
    }
    __syncthreads();
    // ---- stage 1
    for (int it = tid; it < items; it += kThreads) {
      const int i1 = it >> 2, jp = (it & 3) * 2;
      const uint16_t* xr = xs + i1 * L.rs;
      float a0 = 0.f, a1 = 0.f;
      int i2 = 0;
      for (; i2 + 1 < n2; i2 += 2) {
        const uint32_t pr = *(const uint32_t*)(xr + i2);
        const float x0 = widen<BF16>(pr & 0xFFFFu), x1 = widen<BF16>(pr >> 16);
        const float2 p = *(const float2*)(p2s + i2 * kCB + jp);
        const float2 q = *(const float2*)(p2s + (i2 + 1) * kCB + jp);
        a0 = fmaf(x0, p.x, a0); a1 = fmaf(x0, p.y, a1);
        a0 = fmaf(x1, q.x, a0); a1 = fmaf(x1, q.y, a1);
      }
      if (i2 < n2) {
        const float x0 = widen<BF16>(xr[i2]);
        const float2 p = *(const float2*)(p2s + i2 * kCB + jp);
        a0 = fmaf(x0, p.x, a0); a1 = fmaf(x0, p.y, a1);
      }
      *(float2*)(y1 + i1 * kCB + jp) = make_float2(a0, a1);
    }
    __syncthreads();
    // ---- stage 2 and the store
    for (int it = tid; it < items; it += kThreads) {
      const int j1 = it >> 2, jp = (it & 3) * 2;
      float a0 = 0.f, a1 = 0.f;
      for (int i1 = 0; i1 < n1; ++i1) {
        const float p = p1s[i1 * n1 + j1];
        const float2 yv = *(const float2*)(y1 + i1 * kCB + jp);
        a0 = fmaf(p, yv.x, a0); a1 = fmaf(p, yv.y, a1);
      }
      const size_t at = (size_t)m * n + (size_t)j1 * n2 + j0 + jp;
      if (jp < ncol) store_out(Y, at, a0, y_dtype);
      if (jp + 1 < ncol) store_out(Y, at + 1, a1, y_dtype);
    }
  }
}

}  // namespace transform
}  // namespace btc

extern "C" {

btc_status btc_transform(void* stream, const void* X, btc_dtype x_dtype, int32_t M, int32_t n1, int32_t n2,
                         const uint32_t* sign_bits, const float* P1, const float* P2, void* Y, btc_dtype y_dtype) {
  using namespace btc;
  using namespace btc::transform;
  if (!X || !sign_bits || !P1 || !P2 || !Y) return BTC_ERR_NULL;
  if (M <= 0 || n1 <= 0 || n2 <= 0) return BTC_ERR_SHAPE;
  if (n1 > kMaxN1 || n2 > kMaxN2) return BTC_ERR_UNSUPPORTED;
  if (x_dtype != BTC_F16 && x_dtype != BTC_BF16) return BTC_ERR_UNSUPPORTED;
  if (y_dtype != BTC_F16 && y_dtype != BTC_BF16 && y_dtype != BTC_F32) return BTC_ERR_UNSUPPORTED;
  if ((long long)M * n1 * n2 >= (1LL << 40)) return BTC_ERR_SHAPE;
  if (!aligned16(X) || !aligned16(sign_bits) || !aligned16(P1) || !aligned16(P2) || !aligned16(Y)) return BTC_ERR_ALIGN;
  if (X == Y) return BTC_ERR_UNSUPPORTED;    // workgroups read whole rows that others write slices of
  const Layout L = layout_of(n1, n2);
  const int n_cb = (n2 + kCB - 1) / kCB;
  int gy = 1280 / n_cb;                      // about five workgroups per compute unit share the rows
  if (gy < 1) gy = 1;
  if (gy > M) gy = M;
  hipStream_t q = (hipStream_t)stream;
  static bool attr_set[2] = {false, false};  // one-time kernel attributes, not call state
  const int bf = x_dtype == BTC_BF16;
  if (!attr_set[bf]) {
    const void* fn = bf ? (const void*)transform_kernel<true> : (const void*)transform_kernel<false>;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set[bf] = true;
  }
  const dim3 grid(n_cb, gy);
  if (bf)
    transform_kernel<true><<<grid, kThreads, L.total, q>>>((const uint16_t*)X, M, n1, n2, sign_bits, P1, P2, Y,
                                                           (int)y_dtype, L);
  else
    transform_kernel<false><<<grid, kThreads, L.total, q>>>((const uint16_t*)X, M, n1, n2, sign_bits, P1, P2, Y,
                                                            (int)y_dtype, L);
  return launch_status();
}

}  // extern "C"
