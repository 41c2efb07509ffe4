// btc_assign: E-step of the binary codebook clustering (section "Flash and Accurate Binary
// Codebook", step "E-step Assignment"): every +-1 vector of length v goes to its nearest centroid,
//     z_i = argmin_k || b_i - c_k ||^2 = argmin_k 4 d_H(b_i, c_k),   d_H = POPCNT(b_i xor c_k),
// a vector identical to a centroid going to that centroid (distance 0).  Among equally near
// centroids the lowest index wins (the paper leaves ties open; duplicates in the codebook make
// them common).  Integer work, exact.
//
// A thread owns kVec vectors; all threads walk the codebook in the same order, so a codeword is a
// wave-uniform value (scalar loads, no LDS); per (vector, codeword): xor, bit count, and one
// unsigned minimum over the key  distance << 16 | k,  which orders by distance first and index
// second (k < 65536, distance <= 32).  Bound by the vector ALU: about four operations per pair.
#include "btc_internal.h"

namespace btc {
namespace assign {

constexpr int kThreads = 256;
constexpr int kVec = 4;        // vectors per thread

__global__ __launch_bounds__(kThreads) void assign_kernel(const uint32_t* __restrict__ vectors, long long N, int v,
                                                         const uint32_t* __restrict__ codebook, int K,
                                                         int32_t* __restrict__ z, int32_t* __restrict__ dist2) {
  const uint32_t mask = v >= 32 ? 0xFFFFFFFFu : ((1u << v) - 1u);
  const long long first = ((long long)blockIdx.x * kThreads + threadIdx.x) * kVec;
  uint32_t b[kVec], best[kVec];
#pragma unroll
  for (int u = 0; u < kVec; ++u) {
    b[u] = first + u < N ? vectors[first + u] & mask : 0u;
    best[u] = 0xFFFFFFFFu;
  }
  for (int k = 0; k < K; ++k) {
    const uint32_t c = codebook[k] & mask;                     // uniform: a scalar load
#pragma unroll
    for (int u = 0; u < kVec; ++u) {
      const uint32_t key = ((uint32_t)__builtin_popcount(b[u] ^ c) << 16) | (uint32_t)k;
      best[u] = min(best[u], key);
    }
  }
#pragma unroll
  for (int u = 0; u < kVec; ++u) {
    if (first + u < N) {
      z[first + u] = (int32_t)(best[u] & 0xFFFFu);
      if (dist2) dist2[first + u] = (int32_t)(best[u] >> 16) * 4;
    }
  }
}

}  // namespace assign
}  // namespace btc

extern "C" {

btc_status btc_assign(void* stream, const uint32_t* vectors, int64_t N, int32_t v, const uint32_t* codebook,
                      int32_t K, int32_t* z, int32_t* dist2) {
  using namespace btc;
  using namespace btc::assign;
  if (!vectors || !codebook || !z) return BTC_ERR_NULL;
  if (N <= 0) return BTC_ERR_SHAPE;
  if (v < 1 || v > 32 || K < 1 || K > 65536) return BTC_ERR_UNSUPPORTED;
  if (!aligned16(vectors) || !aligned16(codebook) || !aligned16(z) || (dist2 && !aligned16(dist2))) return BTC_ERR_ALIGN;
  const long long per_block = (long long)kThreads * kVec;
  const long long blocks = (N + per_block - 1) / per_block;
  if (blocks > 0x7FFFFFFFLL) return BTC_ERR_SHAPE;
  assign_kernel<<<(unsigned)blocks, kThreads, 0, (hipStream_t)stream>>>(vectors, (long long)N, v, codebook, K, z, dist2);
  return launch_status();
}

}  // extern "C"
