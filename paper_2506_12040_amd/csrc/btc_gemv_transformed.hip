// Decode-time product behind the online activation transform, as ONE call:
//     y = W_hat . (x T),   T = D P,  P = P1 (x) P2
// (section "Learnable Transformation"; "Integration into Transformer Architecture": the activations are
// transformed on the fly in front of every compressed layer).  As two launches -- btc_transform, then btc_gemv --
// the transform of one row costs about as much as the product itself: it is a chain of latencies, not work.
// Here the engine on the 4-bit matrix cores computes the transformed row itself, in every workgroup, from
// factors that were split and laid out once per layer (btc_transform_prepare); see btc_fused_transform.h.
// Settings that engine does not cover run as the two launches, through the head of the workspace.
#include <hip/hip_fp16.h>

#include "btc_fused_transform.h"
#include "btc_internal.h"

namespace btc {
namespace ftr {

// One thread per 16-byte operand pair (hi and lo of eight factors).
__global__ __launch_bounds__(256) void prepare_kernel(int n1, int n2, int IT, int JT, int KS1, int KS2,
                                                      const float* __restrict__ P1, const float* __restrict__ P2,
                                                      uint4* __restrict__ prep) {
  const int n_p2 = JT * KS2 * 64, n_p1 = IT * KS1 * 64;
  for (int it = blockIdx.x * 256 + threadIdx.x; it < n_p2 + n_p1; it += gridDim.x * 256) {
    uint32_t qh[8], ql[8];
    uint4* dst;
    if (it < n_p2) {
      const int ln = it & 63, ks = (it >> 6) % KS2, c = (it >> 6) / KS2;
      const int j2 = 32 * c + (ln & 31), hh = ln >> 5;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int i2 = 16 * ks + 8 * hh + e;
        split2(j2 < n2 ? P2[(size_t)i2 * n2 + j2] : 0.f, qh[e], ql[e]);
      }
      dst = prep + ((size_t)(c * KS2 + ks) * 2) * 64 + ln;
    } else {
      const int jt = it - n_p2;
      const int ln = jt & 63, ks = (jt >> 6) % KS1, a = (jt >> 6) / KS1;
      const int j1 = 32 * a + (ln & 31), hh = ln >> 5;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int i1 = 16 * ks + 8 * (e >> 2) + 4 * hh + (e & 3);
        split2((i1 < n1 && j1 < n1) ? P1[(size_t)i1 * n1 + j1] : 0.f, qh[e], ql[e]);
      }
      dst = prep + (size_t)JT * KS2 * 2 * 64 + ((size_t)(a * KS1 + ks) * 2) * 64 + ln;
    }
    dst[0] = make_uint4(qh[0] | qh[1] << 16, qh[2] | qh[3] << 16, qh[4] | qh[5] << 16, qh[6] | qh[7] << 16);
    dst[64] = make_uint4(ql[0] | ql[1] << 16, ql[2] | ql[3] << 16, ql[4] | ql[5] << 16, ql[6] | ql[7] << 16);
  }
}

static size_t x_region_bytes(const Dims& d) { return (((size_t)d.in * 2) + 255) & ~(size_t)255; }

// The transform of one row as a kernel of its own, from prepared operands: workgroup c computes the 32 output
// columns j2 of block c for all j1 -- wave a < IT tile (a, c) of stage 1, wave IT + a tile (a, c) of stage 2 -- and
// stores them as fp16.  Same arithmetic as the fused prologue (it is the same code with a global destination).
template <int N1, int N2>
__global__ __launch_bounds__(128 * ((N1 + 31) / 32)) void transform_row_kernel(Geo g, const uint16_t* __restrict__ x,
                                                                             uint16_t* __restrict__ y) {
  using FT = Direct<N1, N2>;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.x;
  // the tile numbering of Direct: stage-1 wave a JT + c, stage-2 wave NT + a JT + c
  const int vw = wv < FT::IT ? wv * FT::JT + c : FT::NT + (wv - FT::IT) * FT::JT + c;
  typename FT::Ring ring;
  FT::ring_begin(g, x, vw, lane, ring);
  FT::transform_row(vw, lane, ring, y, (uint4*)smem);
}

template <int N1, int N2>
static btc_status launch_row(hipStream_t q, const Geo& g, const void* x, void* y) {
  using FT = Direct<N1, N2>;
  const size_t lds = exchange_bytes_c(N1, N2);
  static bool attr_set = false;   // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)transform_row_kernel<N1, N2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  transform_row_kernel<N1, N2><<<FT::JT, 128 * FT::IT, lds, q>>>(g, (const uint16_t*)x, (uint16_t*)y);
  return launch_status();
}

// Factor sizes with a row kernel: the pairs of the LLaMA-2 widths with n2 <= 128.
static bool row_kernel_covers(int n1, int n2) {
  return (n1 == 64 && (n2 == 64 || n2 == 80 || n2 == 128)) || (n2 == 128 && (n1 == 86 || n1 == 108));
}
static btc_status transform_row(hipStream_t q, const Geo& g, const void* x, void* y) {
  if (g.n1 == 64 && g.n2 == 64) return launch_row<64, 64>(q, g, x, y);
  if (g.n1 == 64 && g.n2 == 80) return launch_row<64, 80>(q, g, x, y);
  if (g.n1 == 64 && g.n2 == 128) return launch_row<64, 128>(q, g, x, y);
  if (g.n1 == 86 && g.n2 == 128) return launch_row<86, 128>(q, g, x, y);
  if (g.n1 == 108 && g.n2 == 128) return launch_row<108, 128>(q, g, x, y);
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace ftr
}  // namespace btc

extern "C" {

size_t btc_transform_prepared_bytes(int32_t n1, int32_t n2) {
  if (!btc::ftr::geometry_ok(n1, n2) && !btc::ftr::row_kernel_covers(n1, n2)) return 0;
  return btc::ftr::prepared_bytes(n1, n2);
}

btc_status btc_transform_prepare(void* stream, int32_t n1, int32_t n2, const float* P1, const float* P2, void* prepared,
                                 size_t prepared_bytes) {
  using namespace btc;
  if (!P1 || !P2 || !prepared) return BTC_ERR_NULL;
  if (n1 <= 0 || n2 <= 0) return BTC_ERR_SHAPE;
  if (!ftr::geometry_ok(n1, n2) && !ftr::row_kernel_covers(n1, n2)) return BTC_ERR_UNSUPPORTED;
  if (prepared_bytes < ftr::prepared_bytes(n1, n2)) return BTC_ERR_WORKSPACE;
  if (!aligned16(P1) || !aligned16(P2) || !aligned16(prepared)) return BTC_ERR_ALIGN;
  const ftr::Geo g = ftr::make_geo(nullptr, nullptr, n1, n2);
  const int items = (g.JT * g.KS2 + g.IT * g.KS1) * 64;
  ftr::prepare_kernel<<<(items + 255) / 256, 256, 0, (hipStream_t)stream>>>(n1, n2, g.IT, g.JT, g.KS1, g.KS2, P1, P2,
                                                                            (uint4*)prepared);
  return launch_status();
}

size_t btc_gemv_transformed_workspace_bytes(const btc_shape* s) {
  if (!s) return 0;
  const btc::Dims d = btc::dims_of(*s);
  return btc::ftr::x_region_bytes(d) + btc_workspace_bytes(s, 1, 0);
}

btc_status btc_gemv_transformed_multi(void* stream, const btc_shape* s, int32_t count, const uint32_t* const* packed,
                                      const uint32_t* const* codebook, const float* const* alpha,
                                      const float* const* mu, const void* x, int32_t n1, int32_t n2,
                                      const uint32_t* sign_bits, const float* P1, const float* P2, const void* prepared,
                                      void* xt_out, void* const* y, btc_dtype y_dtype, void* workspace,
                                      size_t workspace_bytes) {
  using namespace btc;
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (!packed || !codebook || !alpha || !mu || !x || !sign_bits || !P1 || !P2 || !y) return BTC_ERR_NULL;
  if (count < 1 || count > 4) return BTC_ERR_UNSUPPORTED;
  if (n1 <= 0 || n2 <= 0 || (long long)n1 * n2 != s->in) return BTC_ERR_SHAPE;
  if (y_dtype != BTC_F16 && y_dtype != BTC_F32) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(sign_bits) || !aligned16(P1) || !aligned16(P2) || (prepared && !aligned16(prepared)) ||
      (xt_out && !aligned16(xt_out)))
    return BTC_ERR_ALIGN;
  for (int m = 0; m < count; ++m) {
    if (!packed[m] || !codebook[m] || !alpha[m] || !mu[m] || !y[m]) return BTC_ERR_NULL;
    if (!aligned16(packed[m]) || !aligned16(codebook[m]) || !aligned16(alpha[m]) || !aligned16(mu[m]) || !aligned16(y[m]))
      return BTC_ERR_ALIGN;
  }
  if (xt_out == x) return BTC_ERR_UNSUPPORTED;   // workgroups read x while another one stores the transformed row
  const Dims d = dims_of(*s);
  hipStream_t q = (hipStream_t)stream;
  if (prepared && gemv_fp4_fused_covers(d, n1, n2))
    return gemv_fp4_fused(q, d, count, packed, codebook, alpha, mu, x, n1, n2, sign_bits, prepared, xt_out, y,
                          y_dtype == BTC_F32);
  // the transform as a launch of its own: the row goes through xt_out, or else through the head of the workspace
  const size_t head = xt_out ? 0 : ftr::x_region_bytes(d);
  if (!workspace || workspace_bytes < head + btc_workspace_bytes(s, 1, 0)) return BTC_ERR_WORKSPACE;
  if (!aligned16(workspace)) return BTC_ERR_ALIGN;
  void* xt = xt_out ? xt_out : workspace;
  if (xt == x) return BTC_ERR_UNSUPPORTED;
  if (prepared && ftr::row_kernel_covers(n1, n2))   // the row on the matrix cores, from the prepared operands
    st = ftr::transform_row(q, ftr::make_geo(sign_bits, prepared, n1, n2), x, xt);
  else
    st = btc_transform(stream, x, BTC_F16, 1, n1, n2, sign_bits, P1, P2, xt, BTC_F16);
  if (st != BTC_OK) return st;
  return btc_gemv_multi(stream, s, count, packed, codebook, alpha, mu, xt, y, y_dtype, (unsigned char*)workspace + head,
                        workspace_bytes - head);
}

btc_status btc_gemv_transformed(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                                const float* alpha, const float* mu, const void* x, int32_t n1, int32_t n2,
                                const uint32_t* sign_bits, const float* P1, const float* P2, const void* prepared,
                                void* xt_out, void* y, btc_dtype y_dtype, void* workspace, size_t workspace_bytes) {
  return btc_gemv_transformed_multi(stream, s, 1, &packed, &codebook, &alpha, &mu, x, n1, n2, sign_bits, P1, P2, prepared,
                                    xt_out, &y, y_dtype, workspace, workspace_bytes);
}

}  // extern "C"
