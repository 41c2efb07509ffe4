// btc_gemv: argument checks and engine selection for the decode-time product.
#include <mutex>

#include "btc_internal.h"

// Rough duration in microseconds of one decode pass over the matrix for a single activation
// row (a fixed chain of round trips plus streaming time; fitted to measurements on 7B-shaped
// layers).  Compared with the tiled contraction kernel's own estimate to decide whether a
// batch is served by one pass per row or by one pass of that kernel for all rows.
static double row_pass_us(const btc::Dims& d) { return 3.5 + 1.8e-6 * (double)d.out * d.wpr * 4; }

namespace btc {

// The dispatcher's choice of engine for a shape and a number of activation rows.
static int choose_engine(const Dims& d, int batch) {
  const long long bytes = (long long)d.out * d.wpr * 4;
  int engine = BTC_ENGINE_AUTO;
  {
    // One activation row on the tuned settings (v = 9, 10; 7..10 index bits; rows of at most 30720 weights) and a
    // matrix of 2.5 MiB or more: the engine on the 4-bit matrix cores.  Measured against the engines below on the
    // LLaMA-2 7B / 13B / 70B projection shapes at 0.7 .. 1.11 bit: 7.5 against 10.5 us on 11008 x 4096, 7.8 against
    // 11.5 on 8192 x 8192, 15.0 against 21.6 on 28672 x 8192; level at 13824 x 5120 (8.3 us).  On 5120 x 5120
    // (2.5 MiB) it takes 6.2 us whatever the indices are; the register-resident engine takes 6.2 us on Zipf
    // indices and 7.0 us on uniform ones (its table reads collide less when few codewords dominate).  Below that
    // the longer prologue (table and activation operands are built per workgroup) leaves the register-resident
    // engine ahead (5.4 .. 5.9 against 6.2 us on 4096 x 4096 at 0.9 bit) -- unless the rows are long (6000 weights
    // or more), where that engine and the table engine fall behind from 1 MiB on (2362 x 7266 at 1.0 bit: 9.8 and
    // 8.4 against 7.8 us).
    if (batch == 1 && (bytes >= (5LL << 19) || (bytes >= (1LL << 20) && d.nchunks >= 600)) && gemv_fp4_covers(d))
      engine = BTC_ENGINE_FP4;
    else
    // One row, 9 or 10 index bits, a wide matrix with few enough rows: the single-kernel variant of the
    // matrix-core engine (measured on 4096 x 11008 at 9 bits: 8.6 us against 11.4 for the table engine; at 7 or
    // 8 bits, or with many rows, the other engines stay ahead).
    if (batch == 1 && d.b >= 9 && d.nchunks >= 1024 && d.out <= 6144 && gemv_mfma_one_covers(d))
      engine = BTC_ENGINE_MFMA_ONE;
    else if (gemv_mfma_covers(d, batch) &&
             (batch == 1 ? ((d.b >= 9 && d.nchunks >= 2048 && bytes >= (16LL << 20)) || (d.b == 10 && bytes >= (8LL << 20)))
                         : batch * row_pass_us(d) > gemv_mfma_estimate_us(d, batch)))
      // Several activation rows on a supported setting: one pass of the matrix-core engine serves them all
      // (unless the matrix is so small that a pass per row is still quicker).  A single row goes there too
      // when the matrix is large and so wide that the table engine cannot use its streaming kernel, and for
      // every large matrix with 10-bit indices (128 KB table: one workgroup per compute unit only).
      engine = BTC_ENGINE_MFMA;
    else if (batch > 1 && gemm_tiled_covers(d, batch) && batch * row_pass_us(d) > gemm_tiled_estimate_us(d, batch))
      engine = BTC_ENGINE_TILED;
    else if ((bytes < (3LL << 20) || !lut_engine_covers(d)) && expand_engine_covers(d))
      // Small matrices are bound by the chain of memory round trips: the register-resident engine has the
      // shortest one.  Larger ones are bound by LDS and ALU throughput, where the table engine is lighter.
      engine = BTC_ENGINE_EXPAND;
    else if (lut_engine_covers(d))
      engine = BTC_ENGINE_LUT;
    else if (batch == 1 && gemv_code_covers(d))
      // long vectors or large codebooks (no tuned engine has tables for them): the codebook itself in LDS
      // (4096 x 4096 at v = 16 with 65536 centroids: 32 us with the fallback kernel)
      engine = BTC_ENGINE_CODE;
    else
      engine = BTC_ENGINE_GENERIC;
  }

  return engine;
}

// Whether an engine parks anything in the caller's workspace.
static bool engine_uses_workspace(int engine) {
  return engine == BTC_ENGINE_LUT || engine == BTC_ENGINE_MFMA || engine == BTC_ENGINE_TILED;
}

// Whether btc_gemv on this shape and batch parks anything in (and expects zeros in) its workspace.
bool gemv_auto_uses_workspace(const Dims& d, int batch) { return engine_uses_workspace(choose_engine(d, batch)); }

// One decode call through a chosen engine (engine = BTC_ENGINE_AUTO: the dispatcher's own choice).  A forced
// engine that does not cover the shape or the batch returns BTC_ERR_UNSUPPORTED.
static btc_status gemv_dispatch(int engine, void* stream, const btc_shape* s, const uint32_t* packed,
                                const uint32_t* codebook, const float* alpha, const float* mu, const void* x,
                                int32_t batch, void* y, btc_dtype y_dtype, void* workspace, size_t workspace_bytes) {
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (!packed || !codebook || !alpha || !mu || !x || !y) return BTC_ERR_NULL;
  if (batch < 1 || batch > 16) return BTC_ERR_UNSUPPORTED;
  if (y_dtype != BTC_F16 && y_dtype != BTC_F32) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(packed) || !aligned16(codebook) || !aligned16(alpha) || !aligned16(mu) || !aligned16(x) ||
      !aligned16(y))
    return BTC_ERR_ALIGN;
  hipStream_t q = (hipStream_t)stream;
  const Dims d = dims_of(*s);
  const int y_is_f32 = y_dtype == BTC_F32;
  const size_t ysz = y_is_f32 ? 4 : 2;

  if (engine == BTC_ENGINE_AUTO) engine = choose_engine(d, batch);

  switch (engine) {
    case BTC_ENGINE_MFMA_ONE:
      if (batch != 1 || !gemv_mfma_one_covers(d)) return BTC_ERR_UNSUPPORTED;
      return gemv_mfma_one(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case BTC_ENGINE_MFMA: {
      if (!gemv_mfma_covers(d, batch)) return BTC_ERR_UNSUPPORTED;
      const size_t off = gemv_table_region_bytes(d);
      const size_t need = gemv_mfma_workspace_bytes(d, batch);
      if (!workspace || workspace_bytes < off + need) return BTC_ERR_WORKSPACE;
      if (!aligned16(workspace)) return BTC_ERR_ALIGN;
      return gemv_mfma(q, d, packed, codebook, alpha, mu, x, /*is_bf16=*/0, batch, y, (int)y_dtype, (char*)workspace + off);
    }
    case BTC_ENGINE_TILED: {
      // Decoding the indices is the cost, and the matrix cores take up to 32 rows for the price of one:
      // each index is decoded once for the whole batch.  A k-split call parks partial sums in the workspace
      // (after the table engine's slots of this shape) and zeroes them again in its second pass, so that
      // one zero-filled workspace serves any sequence of calls, whatever their shapes and batch sizes.
      if (!gemm_tiled_covers(d, batch)) return BTC_ERR_UNSUPPORTED;
      const size_t off = gemv_table_region_bytes(d);
      const size_t need = gemm_tiled_workspace_bytes(d, batch);
      if (need > 0) {
        if (!workspace || workspace_bytes < off + need) return BTC_ERR_WORKSPACE;
        if (!aligned16(workspace)) return BTC_ERR_ALIGN;
      }
      return gemm_tiled(q, d, packed, codebook, alpha, mu, x, /*is_bf16=*/0, batch, y, (int)y_dtype,
                        need > 0 ? (char*)workspace + off : nullptr, need, /*clear_workspace=*/1);
    }
    case BTC_ENGINE_EXPAND:
    case BTC_ENGINE_FP4:
      if (engine == BTC_ENGINE_EXPAND ? !expand_engine_covers(d) : !gemv_fp4_covers(d)) return BTC_ERR_UNSUPPORTED;
      for (int m = 0; m < batch; ++m) {   // one pass per activation row
        const void* xm = (const char*)x + (size_t)m * d.in * 2;
        void* ym = (char*)y + (size_t)m * d.out * ysz;
        st = engine == BTC_ENGINE_EXPAND ? gemv_expand(q, d, packed, codebook, alpha, mu, xm, ym, y_is_f32)
                                         : gemv_fp4(q, d, packed, codebook, alpha, mu, xm, ym, y_is_f32);
        if (st != BTC_OK) return st;
      }
      return BTC_OK;
    case BTC_ENGINE_LUT:
      if (!lut_engine_covers(d)) return BTC_ERR_UNSUPPORTED;
      if (!workspace || workspace_bytes < btc_workspace_bytes(s, batch, 0)) return BTC_ERR_WORKSPACE;
      if (!aligned16(workspace)) return BTC_ERR_ALIGN;
      // One pass of the table engine per activation row; the passes share the
      // workspace, which is safe because they are ordered on the stream.
      for (int m = 0; m < batch; ++m) {
        st = gemv_lut(q, d, packed, codebook, alpha, mu, (const char*)x + (size_t)m * d.in * 2,
                      (char*)y + (size_t)m * d.out * ysz, y_is_f32, workspace);
        if (st != BTC_OK) return st;
      }
      return BTC_OK;
    case BTC_ENGINE_CODE:
      if (!gemv_code_covers(d)) return BTC_ERR_UNSUPPORTED;
      for (int m = 0; m < batch; ++m) {   // one pass per activation row
        st = gemv_code(q, d, packed, codebook, alpha, mu, (const char*)x + (size_t)m * d.in * 2,
                       (char*)y + (size_t)m * d.out * ysz, y_is_f32);
        if (st != BTC_OK) return st;
      }
      return BTC_OK;
    case BTC_ENGINE_GENERIC:
      return gemv_generic(q, d, packed, codebook, alpha, mu, x, batch, y, y_is_f32);
  }
  return BTC_ERR_UNSUPPORTED;
}

// ---- the entry point that allocates nothing: scratch memory in a file-scope device array ----------------------
constexpr size_t kStaticScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];     // device address of `scratch` on each GPU, looked up once per device

// Address of this device's copy of the array (the array's name is only a host-side handle).
static btc_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BTC_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BTC_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return BTC_OK;
}

__global__ void clear_scratch_kernel(uint4* p, size_t n16) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace btc

extern "C" {

btc_status btc_gemv_static(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                           const float* alpha, const float* mu, const void* x, int32_t batch, void* y,
                           btc_dtype y_dtype) {
  using namespace btc;
  btc_status st = check_shape(s);
  if (st != BTC_OK) return st;
  if (batch < 1 || batch > 16) return BTC_ERR_UNSUPPORTED;
  const Dims d = dims_of(*s);
  const int engine = choose_engine(d, batch);
  if (!engine_uses_workspace(engine))   // most single-row calls: nothing is parked anywhere
    return gemv_dispatch(engine, stream, s, packed, codebook, alpha, mu, x, batch, y, y_dtype, nullptr, 0);
  const size_t need = btc_workspace_bytes(s, batch, 0);
  if (need > kStaticScratchBytes) return BTC_ERR_WORKSPACE;   // larger than the static array: use btc_gemv
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != BTC_OK) return st;
  // The array keeps whatever the last call left (zeros, unless a call was cut short): what this call's engine
  // expects to be zero is cleared by a small kernel first (no memset node, so that the call can be captured).
  const size_t n16 = (need + 15) / 16;
  clear_scratch_kernel<<<(unsigned)((n16 + 255) / 256 < 1024 ? (n16 + 255) / 256 : 1024), 256, 0, (hipStream_t)stream>>>((uint4*)ws, n16);
  if (launch_status() != BTC_OK) return BTC_ERR_HIP;
  return gemv_dispatch(engine, stream, s, packed, codebook, alpha, mu, x, batch, y, y_dtype, ws, kStaticScratchBytes);
}

btc_status btc_gemv(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* x, int32_t batch, void* y, btc_dtype y_dtype,
                    void* workspace, size_t workspace_bytes) {
  return btc::gemv_dispatch(BTC_ENGINE_AUTO, stream, s, packed, codebook, alpha, mu, x, batch, y, y_dtype, workspace,
                            workspace_bytes);
}

btc_status btc_gemv_engine(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                           const float* alpha, const float* mu, const void* x, int32_t batch, void* y,
                           btc_dtype y_dtype, void* workspace, size_t workspace_bytes, int32_t engine) {
  if (engine < BTC_ENGINE_AUTO || engine > BTC_ENGINE_CODE) return BTC_ERR_UNSUPPORTED;
  return btc::gemv_dispatch(engine, stream, s, packed, codebook, alpha, mu, x, batch, y, y_dtype, workspace,
                            workspace_bytes);
}

btc_status btc_gemv_multi_shapes(void* stream, const btc_shape* const* shapes, int32_t count,
                                 const uint32_t* const* packed, const uint32_t* const* codebook,
                                 const float* const* alpha, const float* const* mu, const void* x, void* const* y,
                                 btc_dtype y_dtype, void* workspace, size_t workspace_bytes) {
  using namespace btc;
  if (!shapes || !packed || !codebook || !alpha || !mu || !x || !y) return BTC_ERR_NULL;
  if (count < 1 || count > 4) return BTC_ERR_UNSUPPORTED;
  if (y_dtype != BTC_F16 && y_dtype != BTC_F32) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(x)) return BTC_ERR_ALIGN;
  int outs[4] = {0, 0, 0, 0}, widest = 0;
  for (int m = 0; m < count; ++m) {
    if (!shapes[m]) return BTC_ERR_NULL;
    const btc_status st = check_shape(shapes[m]);
    if (st != BTC_OK) return st;
    // rows of one length, cut and coded the same way: only the number of rows may differ
    if (shapes[m]->in != shapes[0]->in || shapes[m]->v != shapes[0]->v || shapes[m]->K != shapes[0]->K)
      return BTC_ERR_SHAPE;
    if (!packed[m] || !codebook[m] || !alpha[m] || !mu[m] || !y[m]) return BTC_ERR_NULL;
    if (!aligned16(packed[m]) || !aligned16(codebook[m]) || !aligned16(alpha[m]) || !aligned16(mu[m]) || !aligned16(y[m]))
      return BTC_ERR_ALIGN;
    outs[m] = shapes[m]->out;
    if (shapes[m]->out > shapes[widest]->out) widest = m;
  }
  // one launch where the engine on the 4-bit matrix cores covers the setting (its workgroups are shared out among
  // the matrices in proportion to their rows); else one call per matrix
  const Dims d = dims_of(*shapes[widest]);
  if (count > 1 && gemv_fp4_covers(d))
    return gemv_fp4_multi((hipStream_t)stream, d, count, outs, packed, codebook, alpha, mu, x, y, y_dtype == BTC_F32);
  for (int m = 0; m < count; ++m) {
    const btc_status st = btc_gemv(stream, shapes[m], packed[m], codebook[m], alpha[m], mu[m], x, 1, y[m], y_dtype,
                                   workspace, workspace_bytes);
    if (st != BTC_OK) return st;
  }
  return BTC_OK;
}

btc_status btc_gemv_multi(void* stream, const btc_shape* s, int32_t count, const uint32_t* const* packed,
                          const uint32_t* const* codebook, const float* const* alpha, const float* const* mu,
                          const void* x, void* const* y, btc_dtype y_dtype, void* workspace, size_t workspace_bytes) {
  if (!s) return BTC_ERR_NULL;
  if (count < 1 || count > 4) return BTC_ERR_UNSUPPORTED;
  const btc_shape* shapes[4] = {s, s, s, s};
  return btc_gemv_multi_shapes(stream, shapes, count, packed, codebook, alpha, mu, x, y, y_dtype, workspace,
                               workspace_bytes);
}

}  // extern "C"
