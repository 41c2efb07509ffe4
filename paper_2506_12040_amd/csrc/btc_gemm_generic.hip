// Generic prefill product  Y[M][out] = X[M][in] . W_hat^T  on the matrix cores: any chunk length,
// any index width, ragged shapes.  The tuned kernel (btc_gemm_tiled.hip) covers the common settings.
//
// At many activation rows the layer is a dense contraction, so instead of
// the lookup-and-accumulate scheme of appendix "Binary Codebook LUT-GEMM" the
// index tiles are decoded into +-1 bf16/fp16 tiles in LDS (exact in either
// format) and fed to MFMA with fp32 accumulation; the affine part of the
// dequantisation (Algorithm "Binary Transformation and Compression":
// W_hat = alpha * B_hat + mu) is applied in fp32 afterwards:
//     Y[m][i] = alpha_i * sum_k X[m][k] s[i][k]  +  mu_i * sum_k X[m][k].
// Keeping alpha out of the 16-bit tile avoids rounding it to 8 mantissa bits.
//
// Tiling: a 256-thread workgroup (4 waves, 2 x 2) owns a 128 x 128 output
// tile; each wave owns 64 x 64 = 2 x 2 MFMA 32x32x16 accumulators.  The k
// extent of one LDS tile is a whole number of chunks (16, 8 or 4 of them,
// at most 160 columns), rounded up to a multiple of 16 with zeros.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "btc_internal.h"

namespace btc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kBM = 128, kBN = 128;
constexpr int kKT = 160;           // max k columns per LDS tile
constexpr int kLDK = kKT + 8;      // LDS row stride in elements: 336 B = odd multiple of 16 B
constexpr int kGemmCbLds = 4096;   // codebook entries kept in LDS (16 KB)

template <bool BF16>
__device__ __forceinline__ f32x16 mfma32(const uint4& a, const uint4& b, const f32x16& c) {
  if constexpr (BF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

template <bool BF16, bool CB_LDS>
__global__ __launch_bounds__(256) void gemm_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                   const uint32_t* __restrict__ codebook,
                                                   const float* __restrict__ alpha, const float* __restrict__ mu,
                                                   const uint16_t* __restrict__ X, int M, void* __restrict__ Y,
                                                   int y_dtype, const float* __restrict__ rowsum, int CH) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* Xs = (uint16_t*)smem;                 // [kBM][kLDK]
  uint16_t* Ss = Xs + kBM * kLDK;                 // [kBN][kLDK]
  uint32_t* cb_lds = (uint32_t*)(Ss + kBN * kLDK);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * kBM, n0 = blockIdx.x * kBN;

  if (CB_LDS) {
    for (int k = tid; k < (1 << d.b); k += 256) cb_lds[k] = codebook[k];
  }
  const uint32_t* cb = CB_LDS ? cb_lds : codebook;

  const int kt = CH * d.v;                        // valid k columns per tile
  const int ktp = (kt + 15) & ~15;                // MFMA extent
  const int ntiles = (d.nchunks + CH - 1) / CH;
  const bool vec_ok = (d.in % 8 == 0) && (kt % 8 == 0);
  const uint32_t one2 = BF16 ? 0x3F803F80u : 0x3C003C00u;
  const uint16_t one1 = BF16 ? 0x3F80u : 0x3C00u;

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][c][e] = 0.f;

  for (int tile = 0; tile < ntiles; ++tile) {
    const int k0 = tile * kt;
    __syncthreads();  // previous tile's fragment reads are done (and the codebook is in place)
    // ---- X tile -> LDS (zero beyond M, beyond in, and in the pad columns)
    const int slots = ktp / 8;
    for (int id = tid; id < kBM * slots; id += 256) {
      const int r = id / slots, c = id - r * slots;
      const int m = m0 + r, k = k0 + c * 8;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (m < M) {
        const uint16_t* src = X + (long long)m * d.in + k;
        if (vec_ok && c * 8 + 8 <= kt && k + 8 <= d.in) {
          val = *(const uint4*)src;
        } else {
          uint16_t e[8];
#pragma unroll
          for (int t = 0; t < 8; ++t) e[t] = (c * 8 + t < kt && k + t < d.in) ? src[t] : (uint16_t)0;
          val = make_uint4(e[0] | (uint32_t)e[1] << 16, e[2] | (uint32_t)e[3] << 16,
                           e[4] | (uint32_t)e[5] << 16, e[6] | (uint32_t)e[7] << 16);
        }
      }
      *(uint4*)(Xs + r * kLDK + c * 8) = val;
    }
    // ---- index tile -> +-1 tile in LDS
    for (int id = tid; id < kBN * CH; id += 256) {
      const int r = id / CH, c = id - r * CH;
      const int n = n0 + r, j = tile * CH + c;
      uint16_t* dst = Ss + r * kLDK + c * d.v;
      if (n < d.out && j < d.nchunks) {
        const uint32_t npat = ~cb[field_at(packed + (long long)n * d.wpr, d.wpr, j * d.b, d.b)];
        if ((d.v & 1) == 0) {
          for (int t = 0; t < d.v; t += 2)
            *(uint32_t*)(dst + t) = one2 | ((npat >> t) & 1u) << 15 | ((npat >> (t + 1)) & 1u) << 31;
        } else {
          for (int t = 0; t < d.v; ++t) dst[t] = one1 | (uint16_t)(((npat >> t) & 1u) << 15);
        }
      } else {
        for (int t = 0; t < d.v; ++t) dst[t] = 0;
      }
    }
    for (int id = tid; id < kBN * (ktp - kt); id += 256) {  // pad columns of the sign tile
      const int r = id / (ktp - kt), c = id - r * (ktp - kt);
      Ss[r * kLDK + kt + c] = 0;
    }
    __syncthreads();
    // ---- contraction
    for (int kk = 0; kk < ktp; kk += 16) {
      uint4 af[2], bfr[2];
#pragma unroll
      for (int a = 0; a < 2; ++a)
        af[a] = *(const uint4*)(Xs + (wm * 64 + a * 32 + (lane & 31)) * kLDK + kk + (lane >> 5) * 8);
#pragma unroll
      for (int c = 0; c < 2; ++c)
        bfr[c] = *(const uint4*)(Ss + (wn * 64 + c * 32 + (lane & 31)) * kLDK + kk + (lane >> 5) * 8);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c) acc[a][c] = mfma32<BF16>(af[a], bfr[c], acc[a][c]);
    }
  }

  // ---- epilogue: lane holds output column n (weight row), 16 activation rows per accumulator
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const int n = n0 + wn * 64 + c * 32 + (lane & 31);
    if (n >= d.out) continue;
    const float al = alpha[n], mn = mu[n];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * 64 + a * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (m >= M) continue;
        const float r = al * acc[a][c][e] + mn * rowsum[m];
        const long long o = (long long)m * d.out + n;
        if (y_dtype == BTC_F32) ((float*)Y)[o] = r;
        else if (y_dtype == BTC_BF16) ((__hip_bfloat16*)Y)[o] = __float2bfloat16(r);
        else ((__half*)Y)[o] = __float2half_rn(r);
      }
    }
  }
}

static int gemm_chunks_per_tile(int v) {
  if (16 * v <= kKT) return 16;
  if (8 * v <= kKT) return 8;
  return 4;  // v <= 32 -> 4 v <= 128
}

btc_status gemm_generic(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                        const float* alpha, const float* mu, const void* X, int is_bf16, int M, void* Y,
                        int y_dtype, const float* rowsum) {
  const bool cb_lds = (1 << d.b) <= kGemmCbLds;
  const size_t lds = (size_t)(kBM + kBN) * kLDK * sizeof(uint16_t) + (cb_lds ? sizeof(uint32_t) << d.b : 0);
  const dim3 grid((d.out + kBN - 1) / kBN, (M + kBM - 1) / kBM);
  const int CH = gemm_chunks_per_tile(d.v);
#define BTC_GEMM_LAUNCH(BF, CBL)                                                                              \
  do {                                                                                                         \
    static bool attr_set = false;                                                                              \
    if (!attr_set) {                                                                                           \
      if (hipFuncSetAttribute((const void*)gemm_kernel<BF, CBL>, hipFuncAttributeMaxDynamicSharedMemorySize,   \
                              160 * 1024) != hipSuccess)                                                       \
        return BTC_ERR_HIP;                                                                                    \
      attr_set = true;                                                                                         \
    }                                                                                                          \
    gemm_kernel<BF, CBL><<<grid, 256, lds, q>>>(d, packed, codebook, alpha, mu, (const uint16_t*)X, M, Y,      \
                                                y_dtype, rowsum, CH);                                          \
  } while (0)
  if (is_bf16) {
    if (cb_lds) BTC_GEMM_LAUNCH(true, true); else BTC_GEMM_LAUNCH(true, false);
  } else {
    if (cb_lds) BTC_GEMM_LAUNCH(false, true); else BTC_GEMM_LAUNCH(false, false);
  }
#undef BTC_GEMM_LAUNCH
  return launch_status();
}

}  // namespace btc
