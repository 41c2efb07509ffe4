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
#pragma unroll 8
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

// Short vectors, many of them (N >= 64 * 2^v, v <= 12): there are only 2^v different vectors, so every
// workgroup first assigns all 2^v patterns (the same arithmetic as above, results in LDS as keys
// distance << 16 | k) and then looks its share of the vectors up: N * K pairs become 2^v * K per
// workgroup plus one LDS read per vector, and the call is bound by reading the vectors and writing
// the results.  Identical output by construction.
constexpr int kLutThreads = 1024;

// PPT: patterns per thread (1 for v <= 10, 2^(v - 10) above).  With fewer than 1024 patterns the threads
// that share a pattern split the codebook among them and meet in an LDS minimum (order-independent).
template <int PPT>
__global__ __launch_bounds__(kLutThreads) void assign_lut_kernel(const uint32_t* __restrict__ vectors, long long N, int v,
                                                                const uint32_t* __restrict__ codebook, int K,
                                                                int32_t* __restrict__ z, int32_t* __restrict__ dist2) {
  extern __shared__ uint32_t table[];                          // [2^v] keys
  const uint32_t mask = (1u << v) - 1u;
  const int tid = threadIdx.x;
  const int P = 1 << v;
  if (P < kLutThreads) {
    if (tid < P) table[tid] = 0xFFFFFFFFu;
    __syncthreads();
    const int G = kLutThreads >> v;                            // threads per pattern
    const uint32_t p = (uint32_t)tid & mask;
    const int g = tid >> v;
    const int k_end = (int)((long long)K * (g + 1) / G);
    uint32_t best = 0xFFFFFFFFu;
#pragma unroll 8
    for (int k = (int)((long long)K * g / G); k < k_end; ++k)
      best = min(best, ((uint32_t)__builtin_popcount(p ^ (codebook[k] & mask)) << 16) | (uint32_t)k);
    atomicMin(&table[p], best);
  } else {
    uint32_t best[PPT];
#pragma unroll
    for (int u = 0; u < PPT; ++u) best[u] = 0xFFFFFFFFu;
#pragma unroll 8
    for (int k = 0; k < K; ++k) {
      const uint32_t c = codebook[k] & mask;                   // uniform: a scalar load
#pragma unroll
      for (int u = 0; u < PPT; ++u)
        best[u] = min(best[u], ((uint32_t)__builtin_popcount((uint32_t)(tid + u * kLutThreads) ^ c) << 16) | (uint32_t)k);
    }
#pragma unroll
    for (int u = 0; u < PPT; ++u) table[tid + u * kLutThreads] = best[u];
  }
  __syncthreads();
  const long long step = (long long)gridDim.x * kLutThreads * 4;
  for (long long i = ((long long)blockIdx.x * kLutThreads + tid) * 4; i < N; i += step) {
    if (i + 3 < N) {
      const uint4 b = *(const uint4*)(vectors + i);
      const uint32_t k0 = table[b.x & mask], k1 = table[b.y & mask], k2 = table[b.z & mask], k3 = table[b.w & mask];
      *(int4*)(z + i) = make_int4((int)(k0 & 0xFFFFu), (int)(k1 & 0xFFFFu), (int)(k2 & 0xFFFFu), (int)(k3 & 0xFFFFu));
      if (dist2)
        *(int4*)(dist2 + i) = make_int4((int)(k0 >> 16) * 4, (int)(k1 >> 16) * 4, (int)(k2 >> 16) * 4, (int)(k3 >> 16) * 4);
    } else {
      for (long long j = i; j < N; ++j) {
        const uint32_t key = table[vectors[j] & mask];
        z[j] = (int32_t)(key & 0xFFFFu);
        if (dist2) dist2[j] = (int32_t)(key >> 16) * 4;
      }
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
  if (v <= 12 && N >= (64LL << v)) {
    const long long want = (N + 4 * kLutThreads - 1) / (4 * kLutThreads);
    const unsigned grid = (unsigned)(want < 256 ? want : 256);   // one table per compute unit
    hipStream_t q = (hipStream_t)stream;
    const size_t lds = (size_t)4 << v;
    if (v <= 10) assign_lut_kernel<1><<<grid, kLutThreads, lds, q>>>(vectors, (long long)N, v, codebook, K, z, dist2);
    else if (v == 11) assign_lut_kernel<2><<<grid, kLutThreads, lds, q>>>(vectors, (long long)N, v, codebook, K, z, dist2);
    else assign_lut_kernel<4><<<grid, kLutThreads, lds, q>>>(vectors, (long long)N, v, codebook, K, z, dist2);
    return launch_status();
  }
  const long long per_block = (long long)kThreads * kVec;
  const long long blocks = (N + per_block - 1) / per_block;
  if (blocks > 0x7FFFFFFFLL) return BTC_ERR_SHAPE;
  assign_kernel<<<(unsigned)blocks, kThreads, 0, (hipStream_t)stream>>>(vectors, (long long)N, v, codebook, K, z, dist2);
  return launch_status();
}

}  // extern "C"
