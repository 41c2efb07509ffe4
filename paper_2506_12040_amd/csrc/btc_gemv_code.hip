// Decode-time product for the long-vector settings of the paper's vector-length study (Table
// "Ablation study on vector length / centroids": v = 12 .. 20 and beyond, codebooks of up to 65536
// centroids), one activation row.
//
// With 11 to 16 index bits neither the expanded-codeword tables of the tuned engines nor a table of
// chunk sums fits LDS: the codebook itself (128 KB as 16-bit patterns for v <= 16, or as 32-bit
// patterns up to 32768 centroids) is what LDS can hold, and the blockwise dot product <x_j, C[I_rj]>
// (appendix "Binary Codebook LUT-GEMM") is evaluated from the pattern's bits.  Layout of the work:
//   * a workgroup of 16 waves fills LDS with the codebook and the activation row (fp16) once;
//   * a wave owns one output row at a time; lane l takes chunks l, l + 64, ..: it reads its index
//     from the row's bit stream (consecutive lanes, consecutive fields: coalesced), gathers the
//     pattern from LDS and adds the chunk's activations with the pattern's signs, two at a time:
//     the two sign bits are moved onto the sign positions of a packed fp16 pair, xor-ed in, and
//     the pair is summed in fp32 by a packed dot product with (1, 1);
//   * the index loads of a wave's next row are issued before the current row is reduced.
// A codebook that LDS cannot hold (v > 16 with 16 index bits: 256 KB) is gathered from memory
// instead; it stays in the L2 of every XCD.
// Epilogue: y = alpha * acc + mu * sum(x)  (Algorithm "Binary Transformation and Compression").
#include <hip/hip_fp16.h>

#include <algorithm>
#include <type_traits>

#include "btc_internal.h"

namespace btc {
namespace code {

typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
constexpr int kWaves = 16;
constexpr int kMaxIn = 16384;           // activation row in LDS: 32 KB
constexpr int kMaxSteps = 16;           // chunks per lane and row held in flight

// Sum over the 64 lanes by data-parallel moves (no LDS traffic), valid in lane 63.
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  auto dpp = [](float x, auto ctrl, auto row_mask, auto bound_ctrl) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                                                 decltype(row_mask)::value, 0xF, decltype(bound_ctrl)::value));
  };
  using std::integral_constant;
  v += dpp(v, integral_constant<int, 0xB1>{}, integral_constant<int, 0xF>{}, integral_constant<bool, true>{});    // quad: lane ^ 1
  v += dpp(v, integral_constant<int, 0x4E>{}, integral_constant<int, 0xF>{}, integral_constant<bool, true>{});    // quad: lane ^ 2
  v += dpp(v, integral_constant<int, 0x141>{}, integral_constant<int, 0xF>{}, integral_constant<bool, true>{});   // row_half_mirror
  v += dpp(v, integral_constant<int, 0x140>{}, integral_constant<int, 0xF>{}, integral_constant<bool, true>{});   // row_mirror
  v += dpp(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{}, integral_constant<bool, false>{});  // row_bcast:15
  v += dpp(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{}, integral_constant<bool, false>{});  // row_bcast:31
  return v;
}

// ESZ: bytes of a codebook entry in LDS (2 or 4), 0 = codebook read from memory.  PAIRS: v / 2 as a
// compile-time constant (the chunk's LDS reads are then issued together), 0 = taken from the shape.
template <int ESZ, int PAIRS>
__global__ __launch_bounds__(kWaves * 64) void gemv_code_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                                const uint32_t* __restrict__ codebook,
                                                                const float* __restrict__ alpha,
                                                                const float* __restrict__ mu,
                                                                const uint16_t* __restrict__ x, void* __restrict__ y,
                                                                int y_is_f32) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xs = (uint16_t*)smem;                        // [in rounded up to the chunk grid] fp16, zeros past `in`
  const int xpad = d.nchunks * d.v;
  float* sxp = (float*)(smem + ((xpad * 2 + 15) & ~15));     // [kWaves] partial sums of x
  unsigned char* cb = (unsigned char*)(sxp + kWaves);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_id = blockIdx.x * kWaves + wave, n_waves = gridDim.x * kWaves;
  const uint32_t mask = (1u << d.b) - 1u;
  const int steps = (d.nchunks + 63) >> 6;               // chunks per lane and row

  // index of chunk j of row i; past the row's last chunk: 0 (its activations in LDS are zero)
  auto index_of = [&](int i, int j) -> uint32_t {
    if (j >= d.nchunks) return 0u;
    const uint32_t* row = packed + (size_t)i * d.wpr;
    const uint32_t p = (uint32_t)j * (uint32_t)d.b;
    const uint32_t w = p >> 5, sh = p & 31u;
    const uint32_t lo = row[w];
    const uint32_t hi = (sh + d.b > 32u) ? row[w + 1] : 0u;   // inside the row whenever the field crosses
    return __builtin_amdgcn_alignbit(hi, lo, sh) & mask;
  };
  // the first row's indices fly while LDS is filled
  uint32_t idx[kMaxSteps];
  int i = wave_id;
  if (i < d.out) {
#pragma unroll
    for (int s = 0; s < kMaxSteps; ++s)
      if (s < steps) idx[s] = index_of(i, lane + 64 * s);
  }
  float sx_part = 0.f;                                   // this thread's share of sum(x), the factor of mu
  for (int k = tid; k < xpad / 2; k += kWaves * 64) {    // v is even: whole pairs
    const uint32_t lo = 2 * k < d.in ? x[2 * k] : 0u, hi = 2 * k + 1 < d.in ? x[2 * k + 1] : 0u;
    const uint32_t w = lo | (hi << 16);
    ((uint32_t*)xs)[k] = w;
    const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
    sx_part = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), one, sx_part, false);
  }
  sx_part = wave_sum_to_lane63(sx_part);
  if (lane == 63) sxp[wave] = sx_part;
  // the codebook (inverted: bit set = -1), four entries per load, eight loads in flight per thread
  if (ESZ != 0) {
    const int quads = (1 << d.b) >> 2;
    if (ESZ == 4 && d.b < 2 && tid < (1 << d.b)) ((uint32_t*)cb)[tid] = ~codebook[tid];   // a codebook of two
    for (int k0 = tid; k0 < quads; k0 += 8 * kWaves * 64) {
      uint4 c[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int k = k0 + r * kWaves * 64;
        c[r] = k < quads ? ((const uint4*)codebook)[k] : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int k = k0 + r * kWaves * 64;
        if (k < quads) {
          if (ESZ == 4) ((uint4*)cb)[k] = make_uint4(~c[r].x, ~c[r].y, ~c[r].z, ~c[r].w);
          else ((uint2*)cb)[k] = make_uint2((~c[r].x & 0xFFFFu) | (~c[r].y << 16), (~c[r].z & 0xFFFFu) | (~c[r].w << 16));
        }
      }
    }
  }
  __syncthreads();
  float sx = 0.f;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) sx += sxp[w];

  const int pairs = PAIRS ? PAIRS : d.v >> 1;
  while (i < d.out) {
    // inverted patterns (bit set: -1) of this row's chunks
    uint32_t np[kMaxSteps];
#pragma unroll
    for (int s = 0; s < kMaxSteps; ++s) {
      if (s < steps) {
        if (ESZ == 4) np[s] = ((const uint32_t*)cb)[idx[s]];
        else if (ESZ == 2) np[s] = ((const uint16_t*)cb)[idx[s]];
        else np[s] = ~codebook[idx[s]];
      }
    }
    const int i_next = i + n_waves;
    uint32_t idx_next[kMaxSteps];
    if (i_next < d.out) {
#pragma unroll
      for (int s = 0; s < kMaxSteps; ++s)
        if (s < steps) idx_next[s] = index_of(i_next, lane + 64 * s);
    }
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxSteps; ++s) {
      if (s < steps) {
        const int j = min(lane + 64 * s, d.nchunks - 1);  // (lanes past the last chunk: index 0 times real
        const bool live = lane + 64 * s < d.nchunks;     //  activations -- masked out below)
        const uint32_t* xc = (const uint32_t*)xs + (size_t)j * pairs;
        float a = 0.f;
        auto pair_step = [&](int u, uint32_t xw) {
          const uint32_t n = (np[s] >> (2 * u)) & 3u;
          const uint32_t sg = ((n << 15) | (n << 30)) & 0x80008000u;   // bit 0 -> sign of the low half, bit 1 -> of the high half
          const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
          a = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, xw ^ sg), one, a, false);
        };
        if (PAIRS) {
          uint32_t xw[PAIRS ? PAIRS : 1];
#pragma unroll
          for (int u = 0; u < PAIRS; ++u) xw[u] = xc[u];
#pragma unroll
          for (int u = 0; u < PAIRS; ++u) pair_step(u, xw[u]);
        } else {
          for (int u = 0; u < pairs; ++u) pair_step(u, xc[u]);
        }
        acc += live ? a : 0.f;
      }
    }
    acc = wave_sum_to_lane63(acc);
    if (lane == 63) {
      const float r = alpha[i] * acc + mu[i] * sx;
      if (y_is_f32) ((float*)y)[i] = r;
      else ((__half*)y)[i] = __float2half_rn(r);
    }
    i = i_next;
#pragma unroll
    for (int s = 0; s < kMaxSteps; ++s) idx[s] = idx_next[s];
  }
}

static int entry_bytes(const Dims& d) {
  if ((4LL << d.b) <= 128 * 1024) return 4;
  if (d.v <= 16 && (2LL << d.b) <= 128 * 1024) return 2;
  return 0;
}
static size_t lds_bytes(const Dims& d) {
  return (((size_t)d.nchunks * d.v * 2 + 15) & ~(size_t)15) + kWaves * sizeof(float) + ((size_t)entry_bytes(d) << d.b);
}

}  // namespace code

bool gemv_code_covers(const Dims& d) {
  if (d.v < 2 || (d.v & 1) || d.v > 32 || d.b > 16) return false;
  if (d.in > code::kMaxIn || d.nchunks > 64 * code::kMaxSteps || code::lds_bytes(d) > 160 * 1024) return false;
  if ((long long)d.out * d.wpr * 4 >= (1LL << 31)) return false;
  return true;
}

btc_status gemv_code(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                     const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  using namespace code;
  const int esz = entry_bytes(d);
  const size_t lds = lds_bytes(d);
  const int rows_per_group = kWaves;
  const int grid = std::min(256, (d.out + rows_per_group - 1) / rows_per_group);
#define BTC_CODE_CASE(E, P)                                                                                      \
  if (esz == E && pairs == P) {                                                                                  \
    static bool attr_set = false;                                                                                \
    if (!attr_set) {                                                                                             \
      if (hipFuncSetAttribute((const void*)gemv_code_kernel<E, P>, hipFuncAttributeMaxDynamicSharedMemorySize,   \
                              160 * 1024) != hipSuccess)                                                         \
        return BTC_ERR_HIP;                                                                                      \
      attr_set = true;                                                                                           \
    }                                                                                                            \
    gemv_code_kernel<E, P><<<grid, kWaves * 64, lds, q>>>(d, packed, codebook, alpha, mu, (const uint16_t*)x, y, \
                                                          y_is_f32);                                             \
    return launch_status();                                                                                      \
  }
#define BTC_CODE_ROW(E) BTC_CODE_CASE(E, 6) BTC_CODE_CASE(E, 7) BTC_CODE_CASE(E, 8) BTC_CODE_CASE(E, 9) \
  BTC_CODE_CASE(E, 10) BTC_CODE_CASE(E, 0)
  // the vector lengths of the paper's study are unrolled; every other even length takes the loop
  const int half = d.v >> 1;
  const int pairs = (half >= 6 && half <= 10) ? half : 0;
  BTC_CODE_ROW(4)
  BTC_CODE_ROW(2)
  BTC_CODE_ROW(0)
#undef BTC_CODE_ROW
#undef BTC_CODE_CASE
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace btc
