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
// The workgroup keeps P1 and its slice of P2 in LDS and walks over the rows of X dealt to it; a
// row is staged with its signs applied (a flip of the sign bit: exact).  fp32 accumulation in a
// fixed order: deterministic.  Two shapes of this kernel: for a few rows (decode) the call is
// a chain of latencies, so a workgroup has 1024 threads and every dot product of both stages is
// cut into KS = 4 pieces held by neighbouring lanes, whose sums meet by two cross-lane additions;
// for many rows 256 threads, whole dot products,
// four columns per thread, and the rows are dealt to about five workgroups per compute unit.
// Every global load of a phase is issued before the first one is used.  Many rows of bf16
// activations (prefill) take the matrix-core kernel further down instead.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "btc_internal.h"

namespace btc {
namespace transform {

constexpr int kThreads = 256;
constexpr int kCB = 8;         // columns of P2 per workgroup (4 when a call has very few rows: more workgroups)
constexpr int kMaxN1 = 128;
constexpr int kMaxN2 = 256;

struct Layout {                // byte offsets into dynamic LDS
  int rs;                      // staged row stride in 16-bit elements (even; rs / 2 odd: rows start in different banks)
  int p1, p2, y1, total;
};

static Layout layout_of(int n1, int n2, int KS, int kCB = 8) {
  Layout L;
  L.rs = 2 * (((n2 + 1) / 2) | 1);
  auto up16 = [](int b) { return (b + 15) & ~15; };
  L.p1 = up16(n1 * L.rs * 2);
  L.p2 = L.p1 + up16((n1 * n1 + KS * 32) * 4);                // up to 31 words of padding per piece, here and in Y1
  L.y1 = L.p2 + up16((n2 + KS) * kCB * 4);
  L.total = L.y1 + up16((n1 * kCB + KS * 32) * 4);
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
  } else {                                   // bf16, round to nearest even
    ((__bf16*)Y)[at] = (__bf16)v;
  }
}

// KS: pieces per dot product (threads = 256 KS); CPI: columns per work item; CB: columns per workgroup.
template <bool BF16, int KS, int CPI, int CB>
__global__ __launch_bounds__(kThreads * KS) void transform_kernel(const uint16_t* __restrict__ X, int M, int n1, int n2,
                                                                 const uint32_t* __restrict__ sign_bits,
                                                                 const float* __restrict__ P1,
                                                                 const float* __restrict__ P2, void* __restrict__ Y,
                                                                 int y_dtype, Layout L) {
  constexpr int T = kThreads * KS;
  constexpr int kCB = CB;
  constexpr int IPR = kCB / CPI;             // work items per row index
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xs = (uint16_t*)smem;
  float* p1s = (float*)(smem + L.p1);
  float* p2s = (float*)(smem + L.p2);        // row i2 at i2 * kCB + (i2 / len2) * kCB: a pad per piece, against bank conflicts
  float* y1 = (float*)(smem + L.y1);         // [n1][kCB], row i1 at i1 * kCB + (i1 / len1) * pady
  const int tid = threadIdx.x;
  const int n = n1 * n2;
  const int j0 = blockIdx.x * kCB;
  const int ncol = min(kCB, n2 - j0);
  const int len2 = (((n2 + KS - 1) / KS) + 1) & ~1;   // piece of a stage-1 dot product (even)
  const int len1 = (n1 + KS - 1) / KS;                // piece of a stage-2 dot product
  const float rcp_n2 = 1.0f / (float)n2, rcp_n1 = 1.0f / (float)n1, rcp_len1 = 1.0f / (float)len1;
  // The KS lanes that hold the pieces of one dot product are neighbours (a quad): their sums meet by two
  // cross-lane additions, ((p0 + p1) + (p2 + p3)), and the lane of piece 0 keeps the result.  The rows of P1 and
  // of Y1 that belong to piece ks are shifted by a few words, so that the four lanes of a quad, which read the same
  // column of different pieces, hit different banks: the start of piece ks is 8 ks words (mod 32) after that of
  // piece 0, whatever the sizes.
  const int pad1 = (8 - len1 * n1) & 31, pady = (8 - len1 * kCB) & 31;
  auto quad_sum = [](float a) __attribute__((always_inline)) {
    if constexpr (KS == 4) {
      a += __shfl_xor(a, 1, 64);
      a += __shfl_xor(a, 2, 64);
    }
    return a;
  };
  auto piece_of = [&](int i1) __attribute__((always_inline)) {
    return KS > 1 ? (int)(((float)i1 + 0.5f) * rcp_len1) : 0;  // i1 / len1, exact for these sizes
  };
  const bool x_vec = (n2 & 7) == 0;          // a group of 8 channels stays inside one row of the n1 x n2 view, and
                                             // rows of X start 16-byte aligned

  // A row of X with its signs applied -> LDS (row i1 of the n1 x n2 view at xs + i1 * rs).
  auto stage_x = [&](int m) __attribute__((always_inline)) {
    const uint16_t* xrow = X + (size_t)m * n;
    if (x_vec) {
      constexpr int U = 4;
      const int groups = n >> 3;
      for (int base = tid; base < groups; base += T * U) {
        uint4 v[U];
        uint32_t sw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int g = min(base + u * T, groups - 1);            // past the end: a valid group, not stored
          v[u] = *(const uint4*)(xrow + 8 * g);
          sw[u] = sign_bits[g >> 2];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int g = base + u * T;
          if (g < groups) {
            const int k = 8 * g;
            const int i1 = (int)(((float)k + 0.5f) * rcp_n2);     // exact for k < 2^20
            const int i2 = k - i1 * n2;
            const uint32_t minus = ~(sw[u] >> (k & 31)) & 0xFFu;    // bit e set: channel k + e is flipped
            uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
              w[e] ^= (((minus >> (2 * e)) & 1u) << 15) | (((minus >> (2 * e + 1)) & 1u) << 31);
            uint32_t* dst = (uint32_t*)(xs + i1 * L.rs + i2);       // 4-byte aligned (rs and i2 are even)
            dst[0] = w[0]; dst[1] = w[1]; dst[2] = w[2]; dst[3] = w[3];
          }
        }
      }
    } else {
      for (int k = tid; k < n; k += T) {
        const int i1 = (int)(((float)k + 0.5f) * rcp_n2);
        const int i2 = k - i1 * n2;
        const uint32_t plus = (sign_bits[k >> 5] >> (k & 31)) & 1u;
        xs[i1 * L.rs + i2] = (uint16_t)(xrow[k] ^ (plus ? 0u : 0x8000u));
      }
    }
  };

  // ---- the first row's activations are requested first, then the factors (once per workgroup)
  stage_x(blockIdx.y);
  if ((n2 & 3) == 0) {                       // columns j0 .. j0 + kCB - 1 of a row of P2 are aligned 16-byte pieces
    constexpr int PR = kCB / 4;
    for (int t = tid; t < PR * n2; t += T) {
      const int i2 = t / PR, h = t % PR;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j0 + 4 * h < n2) v = *(const float4*)(P2 + (size_t)i2 * n2 + j0 + 4 * h);
      *(float4*)(p2s + i2 * kCB + (i2 / len2) * kCB + 4 * h) = v;
    }
  } else {
    for (int t = tid; t < n2 * kCB; t += T) {
      const int i2 = t / kCB, jj = t - i2 * kCB;
      p2s[i2 * kCB + (i2 / len2) * kCB + jj] = jj < ncol ? P2[(size_t)i2 * n2 + j0 + jj] : 0.f;
    }
  }
  if ((n1 & 3) == 0) {                       // four consecutive elements stay inside one row of P1
    constexpr int U = 4;
    const int quads = (n1 * n1) >> 2;
    for (int base = tid; base < quads; base += T * U) {
      float4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = *(const float4*)(P1 + 4 * (size_t)min(base + u * T, quads - 1));
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int qd = base + u * T;
        if (qd < quads) {
          const int i1 = (int)(((float)(4 * qd) + 0.5f) * rcp_n1);
          *(float4*)(p1s + 4 * qd + piece_of(i1) * pad1) = v[u];   // pad1 is a multiple of 4 here
        }
      }
    }
  } else {
    for (int t = tid; t < n1 * n1; t += T) {
      const int i1 = (int)(((float)t + 0.5f) * rcp_n1);
      p1s[t + piece_of(i1) * pad1] = P1[t];
    }
  }

  const int items = n1 * IPR * KS;           // item = (row index, group of CPI columns, piece)
  for (int m = blockIdx.y; m < M; m += gridDim.y) {
    if (m != (int)blockIdx.y) {
      __syncthreads();                       // the previous row's readers are done
      stage_x(m);
    }
    __syncthreads();
    // ---- stage 1: piece ks of  Y1[i1][c0 .. c0 + CPI - 1]
    for (int it = tid; it < items; it += T) {
      const int ks = it % KS, rest = it / KS;
      const int c0 = (rest % IPR) * CPI, i1 = rest / IPR;
      const uint16_t* xr = xs + i1 * L.rs;
      const float* pc = p2s + ks * kCB + c0;
      const int lo = ks * len2, hi = min(n2, lo + len2);
      float a[CPI];
#pragma unroll
      for (int c = 0; c < CPI; ++c) a[c] = 0.f;
      int i2 = lo;
      for (; i2 + 1 < hi; i2 += 2) {
        const uint32_t pr = *(const uint32_t*)(xr + i2);
        const float x0 = widen<BF16>(pr & 0xFFFFu), x1 = widen<BF16>(pr >> 16);
        float p[CPI], q[CPI];
        if constexpr (CPI == 4) {
          const float4 pv = *(const float4*)(pc + i2 * kCB), qv = *(const float4*)(pc + (i2 + 1) * kCB);
          p[0] = pv.x; p[1] = pv.y; p[2] = pv.z; p[3] = pv.w;
          q[0] = qv.x; q[1] = qv.y; q[2] = qv.z; q[3] = qv.w;
        } else {
          const float2 pv = *(const float2*)(pc + i2 * kCB), qv = *(const float2*)(pc + (i2 + 1) * kCB);
          p[0] = pv.x; p[1] = pv.y; q[0] = qv.x; q[1] = qv.y;
        }
#pragma unroll
        for (int c = 0; c < CPI; ++c) a[c] = fmaf(x1, q[c], fmaf(x0, p[c], a[c]));
      }
      if (i2 < hi) {
        const float x0 = widen<BF16>(xr[i2]);
#pragma unroll
        for (int c = 0; c < CPI; ++c) a[c] = fmaf(x0, pc[i2 * kCB + c], a[c]);
      }
#pragma unroll
      for (int c = 0; c < CPI; ++c) a[c] = quad_sum(a[c]);
      if (ks == 0) {
        float* dst = y1 + i1 * kCB + piece_of(i1) * pady + c0;
#pragma unroll
        for (int c = 0; c < CPI; ++c) dst[c] = a[c];
      }
    }
    __syncthreads();
    // ---- stage 2: piece ks of  Z[j1][c0 .. c0 + CPI - 1]; a wave's lanes: 16 neighbouring j1 x KS pieces
    for (int it = tid; it < items; it += T) {
      const int ks = it % KS, rest = it / KS;
      const int j1 = rest % n1, c0 = (rest / n1) * CPI;
      const int lo = ks * len1, hi = min(n1, lo + len1);
      const float* pc = p1s + ks * pad1 + j1;
      const float* yc = y1 + ks * pady + c0;
      float a[CPI];
#pragma unroll
      for (int c = 0; c < CPI; ++c) a[c] = 0.f;
      for (int i1 = lo; i1 < hi; ++i1) {
        const float p = pc[i1 * n1];
#pragma unroll
        for (int c = 0; c < CPI; ++c) a[c] = fmaf(p, yc[i1 * kCB + c], a[c]);
      }
#pragma unroll
      for (int c = 0; c < CPI; ++c) a[c] = quad_sum(a[c]);
      if (ks == 0) {
        const size_t at = (size_t)m * n + (size_t)j1 * n2 + j0 + c0;
#pragma unroll
        for (int c = 0; c < CPI; ++c)
          if (c0 + c < ncol) store_out(Y, at + c, a[c], y_dtype);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Many rows of bf16 activations (prefill): the two stages are small dense contractions and
// run on the matrix cores (MFMA 32x32x16 bf16, fp32 accumulate).  A wave owns one row of X
// and one block of 32 columns j2:
//   stage 1:  D1[i1][j2] = sum_i2 (sigma x)[i1][i2] P2[i2][j2]    A = the row itself, read from
//             global memory in operand layout (16 bytes per lane, signs applied in registers);
//             B = P2 from LDS
//   stage 2:  Z[j1][j2]  = sum_i1 P1[i1][j1] D1[i1][j2]           A = P1^T from LDS; B = D1 as it
//             sits in the accumulators: a lane of D1 holds column j2 = lane % 32 and the 16 rows
//             8 (e / 4) + 4 (lane / 32) + e % 4, which is a valid B operand once the contraction
//             index of a 16-row step is permuted the same way in A -- P1^T is staged in that order.
// The fp32 factors and the fp32 D1 enter as sums of three bf16 numbers (24 bits); products whose
// weight is below 2^-24 are dropped, so the result has the accuracy of the fp32 kernel above.
// The activations are bf16 already and enter exactly.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// float -> bf16 bit pattern, round to nearest even (the hardware conversion of gfx950)
__device__ __forceinline__ uint32_t bf16_rne(float v) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)v);
}

// v = p0 + p1 + p2 up to 2^-24 relative, each a bf16 bit pattern
__device__ __forceinline__ void split3(float v, uint32_t& p0, uint32_t& p1, uint32_t& p2) {
  p0 = bf16_rne(v);
  float r = v - __uint_as_float(p0 << 16);
  p1 = bf16_rne(r);
  r -= __uint_as_float(p1 << 16);
  p2 = bf16_rne(r);
}

__device__ __forceinline__ f32x16 mfma32(const uint4& a, const uint4& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// f(integral_constant<int, I>) for I = Begin .. End - 1, fully unrolled
template <int Begin, int End, class F>
__device__ __forceinline__ void static_for_it(F&& f) {
  if constexpr (Begin < End) {
    f(std::integral_constant<int, Begin>{});
    static_for_it<Begin + 1, End>(f);
  }
}

// IT = ceil(n1 / 32): blocks of 32 rows i1 (and of 32 rows j1).  Needs n2 % 16 == 0.
// waves per workgroup: with three or four blocks the operands of P1 fill most of LDS (one workgroup per compute
// unit), so the workgroup is made twice as large to keep two waves per SIMD
template <int IT>
constexpr int mfma_waves() { return IT <= 2 ? 4 : 8; }

// NP: bf16 parts per fp32 operand.  Three (24 bits) for fp32 output; two (16 bits, 2^-17 relative) when the output
// is rounded to fp16 or bf16 anyway (2^-11 / 2^-8): 2 instead of 3 MFMAs per step in stage 1, 3 instead of 6 in stage 2.
template <int IT, int NP>
__global__ __launch_bounds__(64 * mfma_waves<IT>()) void transform_mfma_kernel(const uint16_t* __restrict__ X, int M, int n1, int n2,
                                                                 const uint32_t* __restrict__ sign_bits,
                                                                 const float* __restrict__ P1,
                                                                 const float* __restrict__ P2, void* __restrict__ Y,
                                                                 int y_dtype, int p2_bytes) {
  constexpr int KS1 = 2 * IT;                // 16-row steps of stage 2
  constexpr int NWV = mfma_waves<IT>(), NT = 64 * NWV;
  extern __shared__ __align__(16) unsigned char smem[];
  uint4* P2op = (uint4*)smem;                // [step][part][lane]: B operands of stage 1
  uint4* P1op = (uint4*)(smem + p2_bytes);   // [block j1][step][part][lane]: A operands of stage 2
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const int n = n1 * n2, KS2 = n2 >> 4;
  const int j2 = blockIdx.x * 32 + l32;

  for (int it = tid; it < KS2 * 64; it += NT) {
    const int ks = it >> 6, ln = it & 63, c = blockIdx.x * 32 + (ln & 31), hh = ln >> 5;
    uint32_t q[3][8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i2 = 16 * ks + 8 * hh + e;
      split3(c < n2 ? P2[(size_t)i2 * n2 + c] : 0.f, q[0][e], q[1][e], q[2][e]);
    }
#pragma unroll
    for (int p = 0; p < 3; ++p)
      P2op[(ks * 3 + p) * 64 + ln] = make_uint4(q[p][0] | q[p][1] << 16, q[p][2] | q[p][3] << 16,
                                               q[p][4] | q[p][5] << 16, q[p][6] | q[p][7] << 16);
  }
  for (int it = tid; it < IT * KS1 * 64; it += NT) {
    const int ln = it & 63, ks = (it >> 6) % KS1, jt = (it >> 6) / KS1;
    const int j1 = jt * 32 + (ln & 31), hh = ln >> 5;
    uint32_t q[3][8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i1 = 16 * ks + 8 * (e >> 2) + 4 * hh + (e & 3);   // the row of D1 that element e of a lane's step holds
      split3((i1 < n1 && j1 < n1) ? P1[(size_t)i1 * n1 + j1] : 0.f, q[0][e], q[1][e], q[2][e]);
    }
#pragma unroll
    for (int p = 0; p < 3; ++p)
      P1op[((jt * KS1 + ks) * 3 + p) * 64 + ln] = make_uint4(q[p][0] | q[p][1] << 16, q[p][2] | q[p][3] << 16,
                                                            q[p][4] | q[p][5] << 16, q[p][6] | q[p][7] << 16);
  }
  __syncthreads();

  const uint8_t* sign_bytes = (const uint8_t*)sign_bits;   // byte k / 8 holds the bits of channels k .. k + 7
  // One block of 32 rows i1 at a time: its stage 1 (all steps over i2), the split of its 32 x 32 result, and its
  // share of stage 2 for every block j1 -- so only one block of the intermediate is alive, next to the IT
  // accumulators of the output.  A operands of stage 1 come straight from global memory, PD steps ahead: slot u of
  // the ring holds step ks0 + u of the current chunk of PD steps; once used it is refilled with step ks0 + PD + u
  // of the same block or, in a block's last chunk, with step u of the next block (of the wave's next row after
  // the last block), so the loads always fly during the arithmetic of the block before.
  constexpr int PD = 4;
  const int stride = NWV * gridDim.y;
  auto load_a = [&](int mm, int it, int ks, uint4& a, uint32_t& sg) __attribute__((always_inline)) {
    const int i1 = min(it * 32 + l32, n1 - 1);                 // rows past the end: a valid row, zeroed below
    const int k = i1 * n2 + 16 * ks + 8 * h;
    a = *(const uint4*)(X + (size_t)mm * n + k);
    sg = sign_bytes[k >> 3];
  };
  uint4 ring[PD];
  uint32_t rsg[PD];
  const int m_first = blockIdx.y * NWV + wave;
  if (m_first < M) {
#pragma unroll
    for (int u = 0; u < PD; ++u)
      if (u < KS2) load_a(m_first, 0, u, ring[u], rsg[u]);
  }
  for (int m = m_first; m < M; m += stride) {
    f32x16 z[IT];
#pragma unroll
    for (int jt = 0; jt < IT; ++jt)
#pragma unroll
      for (int e = 0; e < 16; ++e) z[jt][e] = 0.f;
    static_for_it<0, IT>([&](auto it_c) {
      constexpr int it = decltype(it_c)::value;
      f32x16 d1;
#pragma unroll
      for (int e = 0; e < 16; ++e) d1[e] = 0.f;
      const bool row_ok = it * 32 + l32 < n1;
      for (int ks0 = 0; ks0 < KS2; ks0 += PD) {
        const bool last_chunk = ks0 + PD >= KS2;
#pragma unroll
        for (int u = 0; u < PD; ++u) {
          const int ks = ks0 + u;
          if (ks < KS2) {
            const uint32_t minus = ~rsg[u] & 0xFFu;              // bit e set: element e changes sign
            uint4 a = ring[u];
            a.x ^= ((minus & 1u) << 15) | ((minus & 2u) << 30);
            a.y ^= ((minus & 4u) << 13) | ((minus & 8u) << 28);
            a.z ^= ((minus & 16u) << 11) | ((minus & 32u) << 26);
            a.w ^= ((minus & 64u) << 9) | ((minus & 128u) << 24);
            if (!row_ok) a = make_uint4(0u, 0u, 0u, 0u);
            d1 = mfma32(a, P2op[(ks * 3 + 0) * 64 + lane], d1);
            d1 = mfma32(a, P2op[(ks * 3 + 1) * 64 + lane], d1);
            if constexpr (NP == 3) d1 = mfma32(a, P2op[(ks * 3 + 2) * 64 + lane], d1);
          }
          if (ks + PD < KS2) {
            load_a(m, it, ks + PD, ring[u], rsg[u]);
          } else if (last_chunk && u < KS2) {
            if (it + 1 < IT) load_a(m, it + 1, u, ring[u], rsg[u]);
            else if (m + stride < M) load_a(m + stride, 0, u, ring[u], rsg[u]);
          }
        }
      }
      // the block as three bf16 parts, in B-operand form: step s2 takes elements 8 s2 .. 8 s2 + 7
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        uint32_t q[3][8];
#pragma unroll
        for (int e = 0; e < 8; ++e) split3(d1[8 * s2 + e], q[0][e], q[1][e], q[2][e]);
        uint4 y[3];
#pragma unroll
        for (int p = 0; p < 3; ++p)
          y[p] = make_uint4(q[p][0] | q[p][1] << 16, q[p][2] | q[p][3] << 16, q[p][4] | q[p][5] << 16, q[p][6] | q[p][7] << 16);
#pragma unroll
        for (int jt = 0; jt < IT; ++jt) {
          const uint4* ap = P1op + ((jt * KS1 + 2 * it + s2) * 3) * 64 + lane;
          const uint4 a0 = ap[0], a1 = ap[64];
          if constexpr (NP == 3) {                               // small terms first
            z[jt] = mfma32(ap[128], y[0], z[jt]);
            z[jt] = mfma32(a1, y[1], z[jt]);
            z[jt] = mfma32(a0, y[2], z[jt]);
          }
          z[jt] = mfma32(a1, y[0], z[jt]);
          z[jt] = mfma32(a0, y[1], z[jt]);
          z[jt] = mfma32(a0, y[0], z[jt]);
        }
      }
    });
    static_for_it<0, IT>([&](auto jt_c) {
      constexpr int jt = decltype(jt_c)::value;
      const f32x16& zt = z[jt];
      if (j2 < n2) {                                           // one branch on the output type per tile, not per element
        const size_t at0 = (size_t)m * n + (size_t)(jt * 32 + 4 * h) * n2 + j2;
        const int rows_left = n1 - (jt * 32 + 4 * h);            // rows 8 (e / 4) + e % 4 below this count exist
        auto store_tile = [&](auto* out) __attribute__((always_inline)) {
          typedef typename std::remove_pointer<decltype(out)>::type T;
          if ((jt + 1) * 32 <= n1) {                              // a whole block of rows (uniform): no per-element test
#pragma unroll
            for (int e = 0; e < 16; ++e) out[at0 + (size_t)((8 * (e >> 2) + (e & 3)) * n2)] = (T)zt[e];
          } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int r = 8 * (e >> 2) + (e & 3);
              if (r < rows_left) out[at0 + (size_t)(r * n2)] = (T)zt[e];
            }
          }
        };
        if (y_dtype == BTC_BF16) store_tile((__bf16*)Y);
        else if (y_dtype == BTC_F32) store_tile((float*)Y);
        else store_tile((_Float16*)Y);
      }
    });
  }
}

template <int IT, int NP>
static btc_status launch_mfma_np(hipStream_t q, const uint16_t* X, int M, int n1, int n2, const uint32_t* sign_bits,
                              const float* P1, const float* P2, void* Y, int y_dtype) {
  const int p2_bytes = (n2 >> 4) * 3 * 1024;
  const int lds = p2_bytes + IT * 2 * IT * 3 * 1024;
  static bool attr_set = false;              // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)transform_mfma_kernel<IT, NP>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024 - 256) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  const int gx = (n2 + 31) / 32;
  constexpr int NWV = mfma_waves<IT>();
  int gy = (IT <= 2 ? 768 : 256) / gx;       // as many workgroups as stay resident; a wave walks the rows dealt to it
  if (gy > (M + NWV - 1) / NWV) gy = (M + NWV - 1) / NWV;
  if (gy < 1) gy = 1;
  transform_mfma_kernel<IT, NP><<<dim3(gx, gy), 64 * NWV, lds, q>>>(X, M, n1, n2, sign_bits, P1, P2, Y, y_dtype, p2_bytes);
  return launch_status();
}

template <int IT>
static btc_status launch_mfma(hipStream_t q, const uint16_t* X, int M, int n1, int n2, const uint32_t* sign_bits,
                              const float* P1, const float* P2, void* Y, int y_dtype) {
  if (y_dtype == BTC_F32) return launch_mfma_np<IT, 3>(q, X, M, n1, n2, sign_bits, P1, P2, Y, y_dtype);
  return launch_mfma_np<IT, 2>(q, X, M, n1, n2, sign_bits, P1, P2, Y, y_dtype);
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
  hipStream_t q = (hipStream_t)stream;
  if (x_dtype == BTC_BF16 && (n2 & 15) == 0 && M >= 64) {    // prefill on the matrix cores
    const uint16_t* Xm = (const uint16_t*)X;
    switch ((n1 + 31) / 32) {
      case 1: return launch_mfma<1>(q, Xm, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype);
      case 2: return launch_mfma<2>(q, Xm, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype);
      case 3: return launch_mfma<3>(q, Xm, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype);
      default: return launch_mfma<4>(q, Xm, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype);
    }
  }
  int n_cb = (n2 + kCB - 1) / kCB;
  // A few rows: one workgroup of 1024 threads per (column block, row), dot products cut in four.
  // Many rows: 256 threads, and the rows are dealt to about five workgroups per compute unit.
  // Large factors leave room for one workgroup per compute unit only: then the 1024-thread shape serves
  // many rows too (16 waves per compute unit instead of 4).
  const bool few = (long long)M * n_cb <= 512;
  const bool big = layout_of(n1, n2, 1).total > 48 * 1024;
  int KS = (few || big) ? 4 : 1;
  if (KS == 4 && layout_of(n1, n2, 4).total > 160 * 1024 - 256) KS = 1;   // the largest factors: no room for the pads
  // Very few rows: blocks of 4 columns, i.e. twice the workgroups, each with half the arithmetic.
  const int cb = (KS == 4 && few && (long long)M * n_cb <= 128 && n2 >= 8) ? 4 : kCB;
  if (cb == 4) n_cb = (n2 + 3) / 4;
  const Layout L = layout_of(n1, n2, KS, cb);
  if (L.total > 160 * 1024 - 256) return BTC_ERR_UNSUPPORTED;
  int gy = few ? M : big ? 256 / n_cb : 1280 / n_cb;
  if (gy < 1) gy = 1;
  if (gy > M) gy = M;
  static bool attr_set = false;              // one-time kernel attributes, not call state
  if (!attr_set) {
    const void* fns[6] = {(const void*)transform_kernel<false, 4, 2, 8>, (const void*)transform_kernel<true, 4, 2, 8>,
                          (const void*)transform_kernel<false, 4, 2, 4>, (const void*)transform_kernel<true, 4, 2, 4>,
                          (const void*)transform_kernel<false, 1, 4, 8>, (const void*)transform_kernel<true, 1, 4, 8>};
    for (const void* fn : fns)
      if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256) != hipSuccess)
        return BTC_ERR_HIP;
    attr_set = true;
  }
  const bool bf = x_dtype == BTC_BF16;
  const dim3 grid(n_cb, gy);
  const uint16_t* Xp = (const uint16_t*)X;
  if (KS == 4 && cb == 4) {
    if (bf) transform_kernel<true, 4, 2, 4><<<grid, kThreads * 4, L.total, q>>>(Xp, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype, L);
    else transform_kernel<false, 4, 2, 4><<<grid, kThreads * 4, L.total, q>>>(Xp, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype, L);
  } else if (KS == 4) {
    if (bf) transform_kernel<true, 4, 2, 8><<<grid, kThreads * 4, L.total, q>>>(Xp, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype, L);
    else transform_kernel<false, 4, 2, 8><<<grid, kThreads * 4, L.total, q>>>(Xp, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype, L);
  } else {
    if (bf) transform_kernel<true, 1, 4, 8><<<grid, kThreads, L.total, q>>>(Xp, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype, L);
    else transform_kernel<false, 1, 4, 8><<<grid, kThreads, L.total, q>>>(Xp, M, n1, n2, sign_bits, P1, P2, Y, (int)y_dtype, L);
  }
  return launch_status();
}

}  // extern "C"
