// Host-side entry points that touch no device memory: shape arithmetic,
// byte counts, status strings.  (Storage format: Section "Compression
// Analysis" -- ceil(log2 c) index bits per length-v vector.)
#include <algorithm>

#include "btc_internal.h"

namespace btc {

static int ceil_log2(int K) {
  int b = 0;
  while ((1 << b) < K) ++b;
  return b;
}

btc_status check_shape(const btc_shape* s) {
  if (!s) return BTC_ERR_NULL;
  btc_shape t;
  btc_status st = btc_shape_init(&t, s->out, s->in, s->v, s->K);
  if (st != BTC_OK) return st;
  if (t.b != s->b || t.nchunks != s->nchunks || t.words_per_row != s->words_per_row) return BTC_ERR_SHAPE;
  return BTC_OK;
}

}  // namespace btc

extern "C" {

btc_status btc_shape_init(btc_shape* s, int32_t out, int32_t in, int32_t v, int32_t K) {
  if (!s) return BTC_ERR_NULL;
  if (out <= 0 || in <= 0 || v <= 0 || K <= 0) return BTC_ERR_SHAPE;
  if (v > 32 || K < 2 || K > 65536) return BTC_ERR_UNSUPPORTED;
  const int64_t nchunks = ((int64_t)in + v - 1) / v;
  const int b = btc::ceil_log2(K);
  const int64_t wpr = (nchunks * b + 31) / 32;
  // the packed stream stays below 2^40 words; engines that address it with 32-bit byte offsets check
  // for themselves that it is below 2 GiB and leave larger ones to the generic kernels (64-bit indexing)
  if ((int64_t)out * wpr >= ((int64_t)1 << 40)) return BTC_ERR_UNSUPPORTED;
  s->out = out;
  s->in = in;
  s->v = v;
  s->K = K;
  s->b = b;
  s->nchunks = (int32_t)nchunks;
  s->words_per_row = (int32_t)wpr;
  return BTC_OK;
}

size_t btc_packed_bytes(const btc_shape* s) {
  if (!s) return 0;
  return (size_t)s->out * (size_t)s->words_per_row * sizeof(uint32_t);
}

size_t btc_workspace_bytes(const btc_shape* s, int32_t rows, int is_gemm) {
  size_t need = 16;  // range-check flag of btc_pack
  if (!s || rows <= 0) return need;
  const btc::Dims d = btc::dims_of(*s);
  if (is_gemm) {
    need += (((size_t)rows * sizeof(float)) + 15) & ~(size_t)15;  // fp32 row sums of X
    // partial sums of a call that the tiled contraction kernel splits along k
    if (btc::gemm_tiled_covers(d, rows)) need = std::max(need, btc::gemm_tiled_workspace_bytes(d, rows));
    // the sign matrix as bytes, for calls with many rows
    if (btc::gemm_wide_covers(d, rows)) need = std::max(need, btc::gemm_wide_workspace_bytes(d, rows));
    if (btc::gemm_rows_covers(d, rows)) need = std::max(need, btc::gemm_rows_workspace_bytes(d, rows));
    if (rows > 64 && rows <= 128 && btc::gemm_rows_covers(d, 64)) {   // may run as 64 rows + the rest
      need = std::max(need, btc::gemm_rows_workspace_bytes(d, 64));
      if (btc::gemv_mfma_covers(d, 16)) need = std::max(need, btc::gemv_mfma_workspace_bytes(d, 16));
    }
    // a call with few rows may go to the decode engine, 16 rows at a time
    if (rows <= 64 && btc::gemv_mfma_covers(d, rows < 16 ? rows : 16))
      need = std::max(need, btc::gemv_mfma_workspace_bytes(d, rows < 16 ? rows : 16));
  } else {
    // the table engine's slots (zero between calls), then the partial sums of a batched call
    // that goes to the tiled contraction kernel and is split along k
    need = btc::gemv_table_region_bytes(d);
    size_t extra = 0;
    if (rows > 1 && btc::gemm_tiled_covers(d, rows)) extra = btc::gemm_tiled_workspace_bytes(d, rows);
    if (btc::gemv_mfma_covers(d, rows)) extra = std::max(extra, btc::gemv_mfma_workspace_bytes(d, rows));
    need += extra;
  }
  return (need + 255) & ~(size_t)255;
}

const char* btc_status_str(btc_status st) {
  switch (st) {
    case BTC_OK: return "ok";
    case BTC_ERR_NULL: return "null pointer";
    case BTC_ERR_SHAPE: return "bad shape";
    case BTC_ERR_UNSUPPORTED: return "unsupported v, K, batch or dtype";
    case BTC_ERR_ALIGN: return "pointer not 16-byte aligned";
    case BTC_ERR_INDEX_RANGE: return "index outside [0, K)";
    case BTC_ERR_HIP: return "HIP runtime error";
    case BTC_ERR_WORKSPACE: return "workspace missing or too small";
  }
  return "unknown status";
}

}  // extern "C"
