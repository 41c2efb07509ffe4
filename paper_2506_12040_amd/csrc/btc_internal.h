// Internal helpers shared by the HIP translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "btc.h"

namespace btc {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape as the kernels see it (passed by value).
struct Dims {
  int out, in, v, K, b, nchunks, wpr;
};

inline Dims dims_of(const btc_shape& s) {
  return Dims{s.out, s.in, s.v, s.K, s.b, s.nchunks, s.words_per_row};
}

// Re-derive the dependent fields and compare: a shape that was not produced by
// btc_shape_init (or was edited afterwards) is rejected before any launch.
btc_status check_shape(const btc_shape* s);

// Table engine of the decode product (btc_gemv_lut.hip).
bool lut_engine_covers(const Dims& d);
size_t lut_workspace_bytes(const btc_shape& s);
btc_status gemv_lut(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* x, void* y, int y_is_f32, void* ws);
// Register-resident expansion engine for the tuned settings (btc_gemv_expand.hip).
bool expand_engine_covers(const Dims& d);
btc_status gemv_expand(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                       const float* alpha, const float* mu, const void* x, void* y, int y_is_f32);
// Whether btc_gemv's own choice of engine for this shape and batch uses (and wants zero-filled) its workspace.
bool gemv_auto_uses_workspace(const Dims& d, int batch);
// Engine on the 4-bit matrix cores (btc_gemv_fp4.hip): weights as E2M1, activations as E5M2 pieces; one
// kernel, no workspace.
bool gemv_fp4_covers(const Dims& d);
btc_status gemv_fp4(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* x, void* y, int y_is_f32);
// The same engine on up to four matrices applied to the same activation row, in one launch (host arrays of
// device pointers).  outs: the rows of each matrix (all at most d.out; the rest of the shape is d's), or null:
// d.out rows each.
btc_status gemv_fp4_multi(hipStream_t q, const Dims& d, int count, const int* outs, const uint32_t* const* packed,
                          const uint32_t* const* codebook, const float* const* alpha, const float* const* mu,
                          const void* x, void* const* y, int y_is_f32);
// The same engine behind the online activation transform of the row (factors n1 x n1, n2 x n2, n1 n2 = in),
// which every workgroup computes into LDS first; `prepared` from btc_transform_prepare; xt_out: where the
// transformed row is also stored (fp16 [in]), or null; `count` matrices as in gemv_fp4_multi.
bool gemv_fp4_fused_covers(const Dims& d, int n1, int n2);
btc_status gemv_fp4_fused(hipStream_t q, const Dims& d, int count, const uint32_t* const* packed,
                          const uint32_t* const* codebook, const float* const* alpha, const float* const* mu,
                          const void* x, int n1, int n2, const uint32_t* sign_bits, const void* prepared, void* xt_out,
                          void* const* y, int y_is_f32);
// Long vectors and large codebooks, one activation row (btc_gemv_code.hip): the codebook itself in LDS.
bool gemv_code_covers(const Dims& d);
btc_status gemv_code(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                     const float* alpha, const float* mu, const void* x, void* y, int y_is_f32);
// Fallback engine for every other setting (btc_gemv_generic.hip).
btc_status gemv_generic(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                        const float* alpha, const float* mu, const void* x, int batch, void* y, int y_is_f32);

// Matrix-core engine for 1..16 activation rows (btc_gemv_mfma.hip): one pass over the index
// stream for all rows, then a small second pass over partial sums parked in the workspace.
bool gemv_mfma_covers(const Dims& d, int batch);
size_t gemv_mfma_workspace_bytes(const Dims& d, int batch);
double gemv_mfma_estimate_us(const Dims& d, int batch);   // rough duration, for engine selection
btc_status gemv_mfma(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                     const float* alpha, const float* mu, const void* x, int is_bf16, int batch, void* y,
                     int y_dtype, void* workspace);

// Second pass of the engines above and below: y = alpha * (sum of `n_ct` partial-sum planes
// [n_ct][rows][out]) + mu * (sum of `n_ct` row-sum entries, one copy of [n_ct][xstride] per block of
// 256 outputs); clears what it reads.
btc_status skinny_reduce(hipStream_t q, const float* alpha, const float* mu, float* part, float* xpart, int out,
                         int rows, int n_ct, int xstride, void* y, int y_dtype);
// 17..64 activation rows on the same operand scheme (btc_gemm_rows.hip): a workgroup keeps its
// accumulators while it walks its share of the columns, restaging the activations per super-group.
bool gemm_rows_covers(const Dims& d, int M);
size_t gemm_rows_workspace_bytes(const Dims& d, int M);
double gemm_rows_estimate_us(const Dims& d, int M);
btc_status gemm_rows(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                     const float* alpha, const float* mu, const void* X, int is_bf16, int M, void* Y, int y_dtype,
                     void* workspace);

// The same operand scheme for one activation row in a single kernel (16 weight rows per workgroup).
bool gemv_mfma_one_covers(const Dims& d);
btc_status gemv_mfma_one(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                         const float* alpha, const float* mu, const void* x, void* y, int y_is_f32);

// The same scheme on int8 activation codes with the integer matrix cores (btc_gemm_wide_i8.hip):
//   Y = step * (alpha * <signs, codes> + mu * sum(codes)) + lo * wsum
bool gemm_wide_i8_covers(const Dims& d, int M);
size_t gemm_wide_i8_workspace_bytes(const Dims& d, int M);
btc_status gemm_wide_i8(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                        const float* alpha, const float* mu, const float* wsum, const uint8_t* Q, const float* lo,
                        const float* step, int M, void* Y, int y_dtype, void* workspace, size_t workspace_bytes);
// Prefill kernels: the tuned tiling (btc_gemm_tiled.hip) and the generic one (btc_gemm_generic.hip).
bool gemm_tiled_covers(const Dims& d, int M);
btc_status gemm_tiled(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                      const float* alpha, const float* mu, const void* X, int is_bf16, int M, void* Y, int y_dtype,
                      void* workspace, size_t workspace_bytes, int clear_workspace);
size_t gemm_tiled_workspace_bytes(const Dims& d, int M);   // 0 unless the call is split along k
// many activation rows (btc_gemm_wide.hip): the signs expanded once per call into a byte matrix in the workspace,
// contracted by a kernel that streams both operands into LDS with load-to-LDS instructions
bool gemm_wide_covers(const Dims& d, int M);
size_t gemm_wide_workspace_bytes(const Dims& d, int M);
btc_status gemm_wide(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                     const float* alpha, const float* mu, const void* X, int is_bf16, int M, void* Y, int y_dtype,
                     void* workspace, size_t workspace_bytes);
double gemm_tiled_estimate_us(const Dims& d, int M);       // rough duration, for engine selection
// Leading part of a btc_gemv workspace that must stay zero between calls (the table engine's slots).
size_t gemv_table_region_bytes(const Dims& d);
btc_status gemm_generic(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                        const float* alpha, const float* mu, const void* X, int is_bf16, int M, void* Y,
                        int y_dtype, const float* rowsum);

inline btc_status launch_status() {
  return hipGetLastError() == hipSuccess ? BTC_OK : BTC_ERR_HIP;
}

// Extract the b-bit field that starts at bit p of a row's LSB-first stream.
// Never reads word index >= wpr.
__device__ __forceinline__ uint32_t field_at(const uint32_t* __restrict__ row, int wpr, int p, int b) {
  const int w = p >> 5, s = p & 31;
  uint64_t lo = row[w];
  if (s + b > 32 && w + 1 < wpr) lo |= (uint64_t)row[w + 1] << 32;
  return (uint32_t)(lo >> s) & ((1u << b) - 1u);
}

}  // namespace btc
