// btc_pack / btc_unpack: index matrix <-> per-row LSB-first bit stream.
// Integer work only; bit-exact by construction.  (Section "Compression
// Analysis": each length-v vector costs ceil(log2 c) index bits; appendix
// "Binary Codebook LUT-GEMM": index matrix I of shape m x n/v.)
#include "btc_internal.h"

namespace btc {

// One thread per output word.  Word w of a row holds stream bits
// [32w, 32w+32); it gathers every index whose field overlaps that window.
// The thread that owns the word in which a field STARTS range-checks it.
__global__ __launch_bounds__(256) void pack_kernel(Dims d, const int32_t* __restrict__ idx,
                                                   uint32_t* __restrict__ packed,
                                                   uint32_t* __restrict__ flag) {
  const long long total = (long long)d.out * d.wpr;
  for (long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x; g < total;
       g += (long long)gridDim.x * blockDim.x) {
    const int i = (int)(g / d.wpr);
    const int w = (int)(g - (long long)i * d.wpr);
    const int32_t* row = idx + (long long)i * d.nchunks;
    const int lo_bit = w * 32;
    int j = lo_bit / d.b;                          // first field overlapping the window
    uint32_t word = 0;
    bool bad = false;
    for (; j < d.nchunks && j * d.b < lo_bit + 32; ++j) {
      const int32_t code = row[j];
      const int start = j * d.b - lo_bit;          // may be negative: field began in word w-1
      if (start >= 0 && (code < 0 || code >= d.K)) bad = true;
      const uint32_t c = (uint32_t)code & ((1u << d.b) - 1u);
      word |= start >= 0 ? (c << start) : (c >> (-start));
    }
    packed[g] = word;
    if (bad) atomicOr(flag, 1u);
  }
}

// One thread per index.
__global__ __launch_bounds__(256) void unpack_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                     int32_t* __restrict__ idx) {
  const long long total = (long long)d.out * d.nchunks;
  for (long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x; g < total;
       g += (long long)gridDim.x * blockDim.x) {
    const int i = (int)(g / d.nchunks);
    const int j = (int)(g - (long long)i * d.nchunks);
    idx[g] = (int32_t)field_at(packed + (long long)i * d.wpr, d.wpr, j * d.b, d.b);
  }
}

__global__ void clear_flag_kernel(uint32_t* flag) { *flag = 0u; }

static int grid_for(long long total) {
  long long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

}  // namespace btc

extern "C" {

btc_status btc_pack(void* stream, const btc_shape* s, const int32_t* idx, uint32_t* packed,
                    void* workspace, size_t workspace_bytes) {
  btc_status st = btc::check_shape(s);
  if (st != BTC_OK) return st;
  if (!idx || !packed) return BTC_ERR_NULL;
  if (!workspace || workspace_bytes < 16) return BTC_ERR_WORKSPACE;
  if (!btc::aligned16(idx) || !btc::aligned16(packed) || !btc::aligned16(workspace)) return BTC_ERR_ALIGN;
  hipStream_t q = (hipStream_t)stream;
  uint32_t* flag = (uint32_t*)workspace;
  const btc::Dims d = btc::dims_of(*s);
  btc::clear_flag_kernel<<<1, 1, 0, q>>>(flag);
  btc::pack_kernel<<<btc::grid_for((long long)d.out * d.wpr), 256, 0, q>>>(d, idx, packed, flag);
  if (btc::launch_status() != BTC_OK) return BTC_ERR_HIP;
  uint32_t host_flag = 0;
  if (hipMemcpyAsync(&host_flag, flag, sizeof host_flag, hipMemcpyDeviceToHost, q) != hipSuccess) return BTC_ERR_HIP;
  if (hipStreamSynchronize(q) != hipSuccess) return BTC_ERR_HIP;
  return host_flag ? BTC_ERR_INDEX_RANGE : BTC_OK;
}

btc_status btc_unpack(void* stream, const btc_shape* s, const uint32_t* packed, int32_t* idx) {
  btc_status st = btc::check_shape(s);
  if (st != BTC_OK) return st;
  if (!idx || !packed) return BTC_ERR_NULL;
  if (!btc::aligned16(idx) || !btc::aligned16(packed)) return BTC_ERR_ALIGN;
  const btc::Dims d = btc::dims_of(*s);
  btc::unpack_kernel<<<btc::grid_for((long long)d.out * d.nchunks), 256, 0, (hipStream_t)stream>>>(d, packed, idx);
  return btc::launch_status();
}

}  // extern "C"
