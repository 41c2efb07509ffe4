// btc_update: M-step of the binary codebook clustering (section "Flash and Accurate Binary
// Codebook", step "M-step Centroid Update"; the loop over clusters in the algorithm of appendix
// "Binary Codebook Optimization"):  c_k = sign(mean of the vectors assigned to k), a zero mean
// giving +1; a cluster without members keeps its centroid.  Integer work, exact.
//
// Element t of the new centroid is +1 iff  2 * (members with element t = +1) >= members.  So the
// call counts, per cluster, its members and the +1s of every element: v + 1 counters per cluster
// in the caller's workspace.  Pass 1: a workgroup adds up its share of the vectors in an LDS copy
// of the counters (one LDS atomic per set bit and one per vector) and then adds its non-zero
// counters to the workspace.  When the counters of all clusters do not fit LDS (more than 16128)
// the clusters are cut into ranges that do, and every range gets its own workgroups, which read all
// the vectors and count only those of their range: re-reading 8 bytes per vector is far cheaper
// than atomics that go to memory.  Pass 2: one thread per cluster forms the centroid and clears its counters, so the
// workspace is left zero-filled for the next call.  Integer sums: the result does not depend on the
// order of the atomics.
#include <algorithm>

#include "btc_internal.h"

namespace btc {
namespace update {

constexpr int kThreads = 1024;
constexpr int kMaxLdsCounters = 16128;   // 63 KB

__global__ __launch_bounds__(kThreads) void count_kernel(const uint32_t* __restrict__ vectors, const int32_t* __restrict__ z,
                                                        long long N, int v, int K, uint32_t* __restrict__ counts,
                                                        int KR, uint32_t* __restrict__ bad) {
  extern __shared__ uint32_t local[];                          // [KR][v + 1]: clusters k0 .. k0 + KR - 1
  const int W = v + 1;
  const int tid = threadIdx.x;
  const int k0 = blockIdx.y * KR;
  const int kn = min(KR, K - k0);
  for (int t = tid; t < kn * W; t += kThreads) local[t] = 0u;
  __syncthreads();
  const long long step = (long long)gridDim.x * kThreads;
  for (long long i = (long long)blockIdx.x * kThreads + tid; i < N; i += step) {
    const int k = z[i];
    if (k < 0 || k >= K) {                                     // reported by the host after the call; nothing is counted
      *bad = 1u;
      continue;
    }
    if (k < k0 || k >= k0 + kn) continue;                      // another range's cluster
    uint32_t b = vectors[i] & (v >= 32 ? 0xFFFFFFFFu : ((1u << v) - 1u));
    uint32_t* row = local + (size_t)(k - k0) * W;
    atomicAdd(row + v, 1u);
    while (b) {
      const int t = __builtin_ctz(b);
      b &= b - 1u;
      atomicAdd(row + t, 1u);
    }
  }
  __syncthreads();
  for (int t = tid; t < kn * W; t += kThreads) {
    const uint32_t c = local[t];
    if (c) atomicAdd(counts + (size_t)k0 * W + t, c);
  }
}

__global__ __launch_bounds__(256) void vote_kernel(uint32_t* __restrict__ counts, int v, int K,
                                                  uint32_t* __restrict__ codebook, const uint32_t* __restrict__ bad) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= K) return;
  const int W = v + 1;
  uint32_t* row = counts + (size_t)k * W;
  const uint32_t members = row[v];
  uint32_t c = 0u;
  for (int t = 0; t < v; ++t) {
    if (2u * row[t] >= members) c |= 1u << t;                  // sum of +-1 >= 0
    row[t] = 0u;
  }
  row[v] = 0u;
  if (members != 0u && *bad == 0u) codebook[k] = c;
}

__global__ void clear_word_kernel(uint32_t* word) { *word = 0u; }

}  // namespace update
}  // namespace btc

extern "C" {

size_t btc_update_workspace_bytes(int32_t v, int32_t K) {
  if (v < 1 || v > 32 || K < 1 || K > 65536) return 0;
  return ((size_t)K * (size_t)(v + 1) * 4 + 16 + 15) & ~(size_t)15;   // the counters and an error flag
}

btc_status btc_update(void* stream, const uint32_t* vectors, const int32_t* z, int64_t N, int32_t v,
                      uint32_t* codebook, int32_t K, void* workspace, size_t workspace_bytes) {
  using namespace btc;
  using namespace btc::update;
  if (!vectors || !z || !codebook) return BTC_ERR_NULL;
  if (N <= 0) return BTC_ERR_SHAPE;
  if (v < 1 || v > 32 || K < 1 || K > 65536) return BTC_ERR_UNSUPPORTED;
  if (N >= (1LL << 31)) return BTC_ERR_UNSUPPORTED;            // 32-bit counters
  if (!workspace || workspace_bytes < btc_update_workspace_bytes(v, K)) return BTC_ERR_WORKSPACE;
  if (!aligned16(vectors) || !aligned16(z) || !aligned16(codebook) || !aligned16(workspace)) return BTC_ERR_ALIGN;
  hipStream_t q = (hipStream_t)stream;
  uint32_t* counts = (uint32_t*)workspace;
  const size_t n_counters = (size_t)K * (size_t)(v + 1);
  uint32_t* bad = counts + ((n_counters + 3) & ~(size_t)3);
  const int KR = std::min(K, kMaxLdsCounters / (v + 1));       // clusters per range (>= 488)
  const int ranges = (K + KR - 1) / KR;
  long long want = (N + kThreads - 1) / kThreads;
  long long gx = 512 / ranges;                                 // about two workgroups per compute unit in all
  if (gx < 1) gx = 1;
  if (gx > want) gx = want;
  count_kernel<<<dim3((unsigned)gx, (unsigned)ranges), kThreads, (size_t)KR * (v + 1) * 4, q>>>(vectors, z, (long long)N, v, K,
                                                                                              counts, KR, bad);
  if (launch_status() != BTC_OK) return BTC_ERR_HIP;
  vote_kernel<<<(K + 255) / 256, 256, 0, q>>>(counts, v, K, codebook, bad);
  if (launch_status() != BTC_OK) return BTC_ERR_HIP;
  // the one call that waits: an assignment outside [0, K) is an error of the caller's data
  uint32_t flag = 0;
  if (hipMemcpyAsync(&flag, bad, 4, hipMemcpyDeviceToHost, q) != hipSuccess) return BTC_ERR_HIP;
  if (hipStreamSynchronize(q) != hipSuccess) return BTC_ERR_HIP;
  if (flag) {
    clear_word_kernel<<<1, 1, 0, q>>>(bad);                     // the workspace is handed back zero-filled
    return BTC_ERR_INDEX_RANGE;
  }
  return BTC_OK;
}

}  // extern "C"
