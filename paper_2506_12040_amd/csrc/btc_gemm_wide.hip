// Prefill product for many activation rows (512 or more, and enough output tiles to fill the chip):  Y[M][out] = X[M][in] . W_hat^T, in two kernels.
//
// At this size every weight tile is needed by M / 256 workgroups, so decoding it inside each of them
// (btc_gemm_tiled.hip) repeats the table look-ups M / 256 times, and those look-ups and the tile
// writes take more LDS time than the matrix cores leave.  Here the sign matrix B_hat of the layer
// (Algorithm "Binary Transformation and Compression": W_hat = alpha * B_hat + mu) is expanded once
// per call into a scratch matrix of one byte per weight -- the HIGH byte of +-1.0 in the operand's
// 16-bit format -- and the contraction kernel streams tiles of it, like tiles of X, straight from
// memory into LDS with the load-to-LDS instructions (no registers, no LDS writes by a wave, nothing
// to decode).  alpha and mu are applied afterwards in fp32.
//
// Contraction kernel, per workgroup (256 activation rows x BN = 32 NF weight rows, k-tiles of 80):
//   * 4 contraction waves, 64 activation rows each, 2 x NF accumulators of MFMA 32x32x16; both
//     operands come from LDS, read one k-slice ahead of the MFMAs that use them; a weight
//     operand is widened from 8 bytes to 8 16-bit elements by four byte permutes.
//   * 4 loader waves issue the loads of tile t + 2 into the third tile buffer while tile t is
//     contracted; one barrier per tile.
//   * LDS layout is dictated by the load-to-LDS instruction (lane l of a wave writes 16 bytes at
//     base + 16 l), so bank conflicts are avoided by choosing WHICH 16 bytes a lane fetches:
//     activation rows are 160 bytes (10 pieces) with piece p of row r stored at position
//     p ^ ((r / 8) % 2); weight rows are 80 bytes (5 pieces) and read 16 bytes at a time, which
//     is conflict-free as it stands (5 is odd).  A 16-byte weight read covers two k-slices, so
//     inside a block of 32 columns lane half h owns columns 16 h .. 16 h + 15 (first eight: first
//     slice, last eight: second slice), for both operands; the last 16 columns of a tile form a
//     plain slice.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <type_traits>

#include "btc_internal.h"

namespace btc {
namespace wide {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kKT = 80;                 // columns per k-tile
constexpr int kBM = 256;                // activation rows per workgroup
constexpr int kXB = kBM * kKT * 2;      // bytes of an activation tile buffer (no padding)
constexpr int kWBmax = 13 * 1024;       // bytes of a weight tile buffer: 160 x 80, rounded up to whole 1 KB loads
constexpr int kMW = 4, kLW = 4;         // contraction waves, loader waves
constexpr int kXJ = kXB / 1024 / kLW;   // activation loads per loader wave and tile (10)
constexpr uint32_t kOob = 0x80000000u;  // buffer offset that is always out of range
constexpr int kRsrcFlags = 0x00020000;

template <bool BF16>
__device__ __forceinline__ f32x16 mfma32(const uint4& a, const uint4& b, const f32x16& c) {
  if constexpr (BF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// acc + lo + hi of a packed pair of 16-bit floats
template <bool BF16>
__device__ __forceinline__ float pair_sum(uint32_t w, float acc) {
  if constexpr (BF16) {
    const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), one, acc, false);
  } else {
    const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), one, acc, false);
  }
}

__device__ __forceinline__ uint32_t bf16_bits(float v) {
  return (uint32_t)__builtin_bit_cast(uint16_t, __float2bfloat16(v));
}
__device__ __forceinline__ uint32_t f16_bits(float v) {
  return (uint32_t)__builtin_bit_cast(uint16_t, __float2half_rn(v));
}

// LDS traffic inside one wave (writes by some lanes, reads by others): LDS operations of a
// wave complete in order, so waiting for them is enough; the fences pin the compiler.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// 8 weight bytes (the high bytes of +-1.0) -> 8 16-bit operand elements; `low` holds the
// low byte of 1.0 in the operand's format (0x80 for bf16, 0x00 for fp16) in its byte 0.
__device__ __forceinline__ uint4 widen_weights(uint32_t lo, uint32_t hi, uint32_t low) {
  uint4 r;
  r.x = __builtin_amdgcn_perm(lo, low, 0x05000400u);
  r.y = __builtin_amdgcn_perm(lo, low, 0x07000600u);
  r.z = __builtin_amdgcn_perm(hi, low, 0x05000400u);
  r.w = __builtin_amdgcn_perm(hi, low, 0x07000600u);
  return r;
}

// 64 lanes x 16 bytes from memory straight into LDS: lane l's bytes land at dst + 16 l (dst is
// wave-uniform); an out-of-range offset stores zeros.  The host pass of the compiler does not
// know the 16-byte form of the builtin, so it only sees an empty body.
__device__ __forceinline__ void load_to_lds_16(const __amdgpu_buffer_rsrc_t& rsrc, unsigned char* dst, uint32_t voffset,
                                               int soffset) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)dst, 16, voffset, soffset, 0, 0);
#else
  (void)rsrc; (void)dst; (void)voffset; (void)soffset;
#endif
}

constexpr int kRowsAtOnce = 4;      // rows of index words a block of the first kernel holds in LDS
constexpr int kRowWords = 1024;     // words per such row at most (longer rows: read from memory)

// ---- first kernel: the sign matrix as bytes, WB[out][pitch] (pitch = 80 * number of k-tiles; the
// columns past `in` hold the rest of the last chunk's pattern, then zeros: they only ever meet
// zero activations).  One thread per 16 bytes at a time.  The first blocks of the grid (all but
// `expand_blocks`) add up the activation rows instead (one wave per row, fp32): rs[m] = sum_k X[m][k], the factor of mu.
template <bool BF16>
__global__ __launch_bounds__(256) void expand_signs_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                           const uint32_t* __restrict__ codebook,
                                                           unsigned char* __restrict__ WB, int pitch, int expand_blocks,
                                                           const uint16_t* __restrict__ X, int M, float* __restrict__ rs) {
  const int sum_blocks = (int)gridDim.x - expand_blocks;
  if ((int)blockIdx.x < sum_blocks) {                    // (first in the grid: they overlap the expansion)
    const int m = (int)blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (m >= M) return;
    const uint4* row = (const uint4*)(X + (size_t)m * d.in);             // `in` is a multiple of 16 here
    const int n8 = d.in / 8;
    float acc = 0.f;
    for (int base = 0; base < n8; base += 64 * 8) {      // eight loads in flight per lane
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + 64 * u + lane;
        v[u] = i < n8 ? row[i] : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        acc = pair_sum<BF16>(v[u].x, acc);
        acc = pair_sum<BF16>(v[u].y, acc);
        acc = pair_sum<BF16>(v[u].z, acc);
        acc = pair_sum<BF16>(v[u].w, acc);
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) rs[m] = acc;
    return;
  }
  const uint32_t hi_byte = BF16 ? 0x3Fu : 0x3Cu;
  const int pieces = pitch >> 4;
  const uint32_t id = (blockIdx.x - (uint32_t)sum_blocks) * 256u + threadIdx.x;       // out * pitch < 2^31
  const uint32_t mask = (1u << d.b) - 1u;
  if (d.v == 10 && d.b <= 10 && d.wpr <= kRowWords) {
    // Chunk length 10: the 16 columns of a piece lie inside three consecutive chunks.  Their
    // (inverted) patterns, from a table in LDS, are strung together, shifted to the piece's first
    // column, and every 4 bits are spread over the 4 bytes of a word by one 24-bit multiply.
    // A block takes kRowsAtOnce rows at a time: their index words are fetched once, coalesced, into
    // LDS, and the threads pick their three index fields from there (as loads from memory the
    // six words per thread cost more than everything else in this kernel).
    __shared__ uint32_t npat[1024];
    __shared__ uint32_t words[kRowsAtOnce * kRowWords + 1];
    for (int k = threadIdx.x; k < (1 << d.b); k += 256) npat[k] = ~codebook[k] & 0x3FFu;
    const int groups = (d.out + kRowsAtOnce - 1) / kRowsAtOnce;
    for (int grp = (int)blockIdx.x - sum_blocks; grp < groups; grp += expand_blocks) {
      const int row0 = grp * kRowsAtOnce, rows = min(kRowsAtOnce, d.out - row0);
      __syncthreads();                                     // the previous group's words are no longer read
      for (int i = threadIdx.x; i < rows * d.wpr; i += 256) words[i] = packed[(size_t)row0 * d.wpr + i];
      __syncthreads();
      int r = 0, pc = threadIdx.x;
      while (pc >= pieces) { pc -= pieces; ++r; }
      while (r < rows) {
        const uint32_t* prow = words + r * d.wpr;
        const int j0 = (pc * 16) / 10, t0 = pc * 16 - 10 * j0;
        uint32_t bits = 0u;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
          const int j = j0 + u;
          if (j < d.nchunks) {                             // (past the last chunk: +1 bytes, they meet zero activations)
            const uint32_t bit = (uint32_t)j * (uint32_t)d.b;
            const uint32_t w0 = bit >> 5, sh = bit & 31u;
            const uint32_t lo = prow[w0];
            const uint32_t hi = prow[w0 + 1];              // (one word past the row at most: inside `words`, shifted out)
            bits |= npat[__builtin_amdgcn_alignbit(hi, lo, sh) & mask] << (10 * u);
          }
        }
        const uint32_t n16 = bits >> t0;
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
          w[q] = (((__umul24((n16 >> (4 * q)) & 0xFu, 0x204081u)) & 0x01010101u) << 7) | (hi_byte * 0x01010101u);
        *(uint4*)(WB + (size_t)(row0 + r) * pitch + (size_t)pc * 16) = make_uint4(w[0], w[1], w[2], w[3]);
        pc += 256;
        while (pc >= pieces) { pc -= pieces; ++r; }
      }
    }
    return;
  }
  if (d.v == 10 && d.b <= 10) {
    // The same for rows too long for the LDS copy: index words straight from memory.
    __shared__ uint32_t npat[1024];
    for (int k = threadIdx.x; k < (1 << d.b); k += 256) npat[k] = ~codebook[k] & 0x3FFu;
    __syncthreads();
    const uint32_t total = (uint32_t)d.out * (uint32_t)pieces;
    for (uint32_t it = id; it < total; it += (uint32_t)expand_blocks * 256u) {
    const int row = (int)(it / (uint32_t)pieces), pc = (int)(it - (uint32_t)row * (uint32_t)pieces);
    const uint32_t* prow = packed + (size_t)row * d.wpr;
    const int j0 = (pc * 16) / 10, t0 = pc * 16 - 10 * j0;
    uint32_t idx[3];
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      const int j = j0 + u;
      idx[u] = 0xFFFFFFFFu;
      if (j < d.nchunks) {                               // (past the last chunk: +1 bytes, they meet zero activations)
        const uint32_t bit = (uint32_t)j * (uint32_t)d.b;
        const uint32_t w0 = bit >> 5, sh = bit & 31u;
        const uint32_t lo = prow[w0];
        const uint32_t hi = (sh + d.b > 32u) ? prow[w0 + 1] : 0u;   // inside the row whenever the field crosses
        idx[u] = __builtin_amdgcn_alignbit(hi, lo, sh) & mask;
      }
    }
    uint32_t bits = 0u;
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (idx[u] != 0xFFFFFFFFu) bits |= npat[idx[u]] << (10 * u);
    const uint32_t n16 = bits >> t0;
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
      w[q] = (((__umul24((n16 >> (4 * q)) & 0xFu, 0x204081u)) & 0x01010101u) << 7) | (hi_byte * 0x01010101u);
    *(uint4*)(WB + (size_t)row * pitch + (size_t)pc * 16) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    return;
  }
  for (uint32_t it = id; it < (uint32_t)d.out * (uint32_t)pieces; it += (uint32_t)expand_blocks * 256u) {
  const int row = (int)(it / (uint32_t)pieces), pc = (int)(it - (uint32_t)row * (uint32_t)pieces);
  const uint32_t* prow = packed + (size_t)row * d.wpr;
  int k = pc * 16;
  int j = k / d.v, t = k - j * d.v;
  uint32_t pat = 0u;
  bool have = false;
  uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    if (!have) {
      if (j < d.nchunks) {
        const long long bit = (long long)j * d.b;
        const int w0 = (int)(bit >> 5), sh = (int)(bit & 31);
        const uint32_t lo = prow[w0];
        const uint32_t hi = (sh + d.b > 32) ? prow[w0 + 1] : 0u;   // inside the row whenever the field crosses
        pat = codebook[__builtin_amdgcn_alignbit(hi, lo, (uint32_t)sh) & mask];
      }
      have = true;
    }
    uint32_t byte = 0u;
    if (j < d.nchunks) byte = hi_byte | ((((pat >> t) & 1u) ^ 1u) << 7);
    w[e >> 2] |= byte << (8 * (e & 3));
    if (++t == d.v) {
      t = 0;
      ++j;
      have = false;
    }
  }
  *(uint4*)(WB + (size_t)row * pitch + (size_t)pc * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

#ifdef BTC_WIDE_STAMPS
__device__ unsigned long long g_stamps[3 * 2 * 16];
// thread 0 of a loader wave (role 1) and of contraction wave 0 (role 0), in the first, middle and last workgroup
#define WSTAMP(role, i)                                                                              \
  do {                                                                                               \
    if (lane == 0 && (blockIdx.x == 0 || blockIdx.x == gridDim.x / 2 || blockIdx.x == gridDim.x - 9))  \
      g_stamps[((blockIdx.x == 0 ? 0 : (blockIdx.x == gridDim.x - 9 ? 2 : 1)) * 2 + (role)) * 16 + (i)] = wall_clock64(); \
  } while (0)
#else
#define WSTAMP(role, i)
#endif

// ---- second kernel: the contraction
template <int NF, bool BF16>
__global__ __launch_bounds__((kMW + kLW) * 64) void gemm_wide_kernel(
    int in, int out, const unsigned char* __restrict__ WB, int pitch, const float* __restrict__ alpha,
    const float* __restrict__ mu, const uint16_t* __restrict__ X, const float* __restrict__ rs_all, int M,
    void* __restrict__ Y, int y_dtype, int m_blocks, int n_blocks, int gm) {
  constexpr int BN = 32 * NF;
  constexpr int kWJ = (BN * 5 + 63) / 64;                // weight loads (of 1 KB) per tile
  extern __shared__ __align__(16) unsigned char smem[];
  // LDS: activation tiles [3][256 rows][160 bytes] at 0, then weight tiles [3][kWBmax]
  unsigned char* const WT = smem + 3 * kXB;

  // ---- workgroup -> (m block, n block); consecutive ids go to consecutive XCDs
  int mb, nb;
  {
    const int L = blockIdx.x;
    // Workgroup L runs on XCD L % 8.  The XCDs form a grid of gm x gn (gm gn = 8): XCD (xm, xn) takes the
    // m blocks = xm (mod gm) and the n blocks = xn (mod gn), so the chip reads the weight bytes gm times and the
    // activations gn times (through eight separate L2 caches); the host picks the split with the least traffic.
    // Consecutive workgroups of an XCD share their weight tile.
    const int x = L & 7, sq = L >> 3;
    const int gn = 8 / gm;
    const int xm = x % gm, xn = x / gm;
    const int pm = (m_blocks + gm - 1) / gm;
    mb = xm + gm * (sq % pm);
    nb = xn + gn * (sq / pm);
    if (mb >= m_blocks || nb >= n_blocks) return;
  }
  const int m0 = mb * kBM, n0 = nb * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nt = pitch / kKT;

  if (wave >= kMW) {
    // =============================== loader waves ===============================
    const int lw = wave - kMW;
    const __amdgpu_buffer_rsrc_t rX =
        __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, (int)((long long)M * in * 2), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rW =
        __builtin_amdgcn_make_buffer_rsrc((void*)WB, 0, (int)((long long)out * pitch), kRsrcFlags);
    // Activation load i of this wave fills positions 64 (kXJ lw + i) + lane of the tile (10 per row).
    // Rows m >= M need no test of their own: X is row-major, so they lie past the end of the
    // buffer and the hardware range check makes the load store zeros.
    uint32_t xv[kXJ];                                    // byte offset of this lane's piece in tile 0
    int xp[kXJ];                                         // its piece number (for the ragged last tile)
#pragma unroll
    for (int i = 0; i < kXJ; ++i) {
      const int g = 64 * (kXJ * lw + i) + lane;
      const int row = g / 10, pos = g - 10 * row;
      xp[i] = pos ^ ((row >> 3) & 1);
      xv[i] = (uint32_t)(((long long)(m0 + row) * in + 8 * xp[i]) * 2);
    }
    // Weight load i (i = lw, lw + 4, ..) fills positions 64 i + lane of the tile (5 per row); rows past
    // the end of the matrix lie past the end of the scratch matrix: zeros.
    constexpr int kWI = (kWJ + kLW - 1) / kLW;
    uint32_t wv[kWI];
#pragma unroll
    for (int i = 0; i < kWI; ++i) {
      const int g = 64 * (lw + kLW * i) + lane;
      const int row = g / 5, pos = g - 5 * row;
      wv[i] = (lw + kLW * i < kWJ && row < BN) ? (uint32_t)((long long)(n0 + row) * pitch + 16 * pos) : kOob;
    }
    auto issue = [&](int t, int buf) {
      if (t >= nt) return;                               // (uniform)
      unsigned char* const xb = smem + buf * kXB + kXJ * lw * 1024;
      if ((t + 1) * kKT <= in) {                         // the whole tile lies inside the rows: scalar column offset
#pragma unroll
        for (int i = 0; i < kXJ; ++i)
          load_to_lds_16(rX, xb + i * 1024, xv[i], t * kKT * 2);
      } else {
        // `in` is a multiple of 16 for this kernel, so a piece lies wholly inside or outside the row
#pragma unroll
        for (int i = 0; i < kXJ; ++i) {
          const uint32_t off = (t * kKT + 8 * xp[i] + 8 > in) ? kOob : xv[i] + (uint32_t)(t * kKT) * 2u;
          load_to_lds_16(rX, xb + i * 1024, off, 0);
        }
      }
#pragma unroll
      for (int i = 0; i < kWI; ++i)
        if (lw + kLW * i < kWJ)                          // (uniform)
          load_to_lds_16(rW, WT + buf * kWBmax + (lw + kLW * i) * 1024, wv[i], t * kKT);
    };
    // Tile t lives in buffer t % 3.  Its loads are issued right after the barrier that ends tile
    // t - 3 (whose buffer it takes over) and must have landed at the barrier that ends tile t - 1.
    if (lw == 0) WSTAMP(1, 0);
    issue(0, 0);
    issue(1, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)
    if (lw == 0) WSTAMP(1, 1);
    __builtin_amdgcn_s_barrier();                        // tiles 0 and 1 are in LDS
    int buf = 2;
    for (int t = 0; t < nt; ++t) {
      issue(t + 2, buf);
      buf = buf == 2 ? 0 : buf + 1;
      // everything but the loads just issued has landed (a wave's loads complete in order)
      static_assert(kXJ + kWI <= 15, "the count must fit the low four bits of the wait");
      if (t + 2 >= nt) __builtin_amdgcn_s_waitcnt(0x0F70);                       // vmcnt(0)
      else if (lw + kLW * (kWI - 1) < kWJ) __builtin_amdgcn_s_waitcnt(0x0F70 | (kXJ + kWI));
      else __builtin_amdgcn_s_waitcnt(0x0F70 | (kXJ + kWI - 1));
      __builtin_amdgcn_s_barrier();                      // tile t consumed, tile t + 1 in LDS
    }
    return;
  }

  // ================================= contraction waves =================================
  if (m0 + wave * 64 >= M) {                             // no activation rows for this wave: keep the barriers only
    __syncthreads();
    for (int t = 0; t < nt; ++t) __syncthreads();
    return;
  }
  __builtin_amdgcn_s_setprio(2);                         // the matrix pipe is the bottleneck: issue these first
  const int h = lane >> 5, l32 = lane & 31;
  f32x16 acc[2][NF];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < NF; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][c][e] = 0.f;

  // Steps of a tile: 0, 1 = the two slices of columns 0..31; 2, 3 = of columns 32..63; 4 = columns
  // 64..79.  Activation piece (8 columns) of lane half h in step s: 4 (s / 2) + 2 h + (s % 2) for
  // s < 4, 8 + h for s = 4; stored at that number ^ swz, swz = (row / 8) % 2.
  const int swz = (l32 >> 3) & 1;
  // two per-lane addresses serve all steps (the rest are instruction offsets): even steps (odd
  // steps: the neighbouring piece, bit 4 flipped) and step 4
  const uint32_t a_base = (uint32_t)((wave * 64 + l32) * (kKT * 2));
  const uint32_t a_even = a_base + (uint32_t)((2 * h + swz) * 16);
  const uint32_t a_last = a_base + (uint32_t)((8 + (h ^ swz)) * 16);
  const uint32_t b_pair = (uint32_t)(3 * kXB + l32 * kKT + 16 * h);   // + c * 32 * 80 + 16 s  (s = 0, 2)
  const uint32_t b_last = (uint32_t)(3 * kXB + l32 * kKT + 64 + 8 * h);
  const uint32_t low = BF16 ? 0x80u : 0x00u;
  uint4 afr[2][2];                                       // [register set][fragment]
  uint4 bq[2][NF];                                       // [register set][weight block]: 16 bytes = two slices
  uint4 bw[2];                                           // widened weights, two sets in turn
  auto read_a = [&](int set, int xoff, int s) {
    const uint32_t at = (uint32_t)xoff + (s == 4 ? a_last : (s & 1) ? (a_even ^ 16u) : a_even);
#pragma unroll
    for (int a = 0; a < 2; ++a)
      afr[set][a] = *(const uint4*)(smem + at + a * 32 * (kKT * 2) + (s < 4 ? 64 * (s >> 1) : 0));
  };
  auto read_b = [&](int set, int woff, int s) {          // s = 0, 2: 16 bytes; s = 4: 8 bytes
#pragma unroll
    for (int c = 0; c < NF; ++c) {
      if (s < 4) {
        bq[set][c] = *(const uint4*)(smem + ((uint32_t)woff + b_pair) + c * 32 * kKT + 16 * s);
      } else {
        const uint2 v = *(const uint2*)(smem + ((uint32_t)woff + b_last) + c * 32 * kKT);
        bq[set][c].x = v.x;
        bq[set][c].y = v.y;
      }
    }
  };
  auto b_words = [&](int set, int c, int s, uint32_t& lo, uint32_t& hi) {
    if (s & 1) { lo = bq[set][c].z; hi = bq[set][c].w; }
    else { lo = bq[set][c].x; hi = bq[set][c].y; }
  };
  if (wave == 0) WSTAMP(0, 0);
  __syncthreads();                                       // tiles 0 and 1 are in LDS
  if (wave == 0) WSTAMP(0, 1);
  read_a(0, 0, 0);
  read_b(0, 0, 0);
  // Register sets: activations alternate per step, weights per 16-byte read (steps 0, 2, 4); a tile
  // has an odd number of either, so both follow the tile's parity P.  Weight set of steps 0, 1 and
  // 4: P; of steps 2, 3: P ^ 1; the next tile's first read goes to P ^ 1.
  auto tile = [&](int xoff, int woff, int xnext, int wnext, bool has_next, auto parity) {
    constexpr int P = decltype(parity)::value;
#pragma unroll
    for (int s = 0; s < 5; ++s) {
      const int aset = (P + s) & 1;
      const int bset = (s == 2 || s == 3) ? (P ^ 1) : P;
      __builtin_amdgcn_sched_barrier(0);
      if (s < 4) {
        read_a(aset ^ 1, xoff, s + 1);
        if (s == 1) read_b(P ^ 1, woff, 2);
        if (s == 3) read_b(P, woff, 4);
      } else {
        __syncthreads();                                 // this tile is in registers; the next one is in LDS
        if (has_next) {
          read_a(aset ^ 1, xnext, 0);
          read_b(P ^ 1, wnext, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (s == 0) {
        uint32_t lo, hi;
        b_words(bset, 0, s, lo, hi);
        bw[0] = widen_weights(lo, hi, low);
      }
#pragma unroll
      for (int c = 0; c < NF; ++c) {
        // order pinned: the permutes for the next block are issued in the shadow of this block's
        // two MFMAs and write registers no MFMA in flight reads
        const int g = s * NF + c;
        __builtin_amdgcn_sched_barrier(0);
        acc[0][c] = mfma32<BF16>(afr[aset][0], bw[g & 1], acc[0][c]);
        __builtin_amdgcn_sched_barrier(0);
        if (c + 1 < NF) {
          uint32_t lo, hi;
          b_words(bset, c + 1, s, lo, hi);
          bw[(g + 1) & 1] = widen_weights(lo, hi, low);
        } else if (s + 1 < 5) {
          const int nset = (s + 1 == 2 || s + 1 == 3) ? (P ^ 1) : P;
          uint32_t lo, hi;
          b_words(nset, 0, s + 1, lo, hi);
          bw[(g + 1) & 1] = widen_weights(lo, hi, low);
        }
        __builtin_amdgcn_sched_barrier(0);
        acc[1][c] = mfma32<BF16>(afr[aset][1], bw[g & 1], acc[1][c]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  {
    int b0 = 0;                                          // buffer of the current tile
    for (int t = 0; t < nt; t += 2) {
      const int b1 = b0 == 2 ? 0 : b0 + 1, b2 = b1 == 2 ? 0 : b1 + 1;
      tile(b0 * kXB, b0 * kWBmax, b1 * kXB, b1 * kWBmax, t + 1 < nt, std::integral_constant<int, 0>{});
      if (t + 1 < nt) tile(b1 * kXB, b1 * kWBmax, b2 * kXB, b2 * kWBmax, t + 2 < nt, std::integral_constant<int, 1>{});
      b0 = b2;
    }
  }

  if (wave == 0) WSTAMP(0, 2);
  // ---- epilogue.  After the last barrier the tile buffers are free; each wave uses a part of
  // them to turn its accumulators (lane = weight row n, 16 activation rows per register set)
  // into rows of Y, so that a lane stores 4 consecutive outputs at once.
  constexpr int TS = BN + 4;                                   // floats per staged row
  float* Tw = (float*)smem + wave * (32 * TS);                 // 32 rows x BN of this wave
  float* rsb = (float*)smem + kMW * (32 * TS) + wave * 64;     // its 64 row sums
  float al[NF], mn[NF];
#pragma unroll
  for (int c = 0; c < NF; ++c) {
    const int n = n0 + c * 32 + l32;
    al[c] = n < out ? alpha[n] : 0.f;
    mn[c] = n < out ? mu[n] : 0.f;
  }
  // activation row sums of this wave's 64 rows (from the first kernel); every lane then picks up the 32 it needs
  {
    const int m = m0 + wave * 64 + lane;
    rsb[lane] = m < M ? rs_all[m] : 0.f;
  }
  wave_lds_sync();
  if (wave == 0) WSTAMP(0, 3);
  const bool vec = (out & 3) == 0;                             // 4 outputs of a row are aligned and inside
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int mrow0 = m0 + wave * 64 + a * 32;
    float rs[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 v = *(const float4*)(rsb + a * 32 + 8 * g + 4 * h);
      rs[4 * g + 0] = v.x; rs[4 * g + 1] = v.y; rs[4 * g + 2] = v.z; rs[4 * g + 3] = v.w;
    }
#pragma unroll
    for (int c = 0; c < NF; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e)
        Tw[(8 * (e >> 2) + 4 * h + (e & 3)) * TS + c * 32 + l32] = al[c] * acc[a][c][e] + mn[c] * rs[e];
    wave_lds_sync();
    if (vec) {
      // The staged rows leave in batches: all LDS reads of a batch are issued, then its stores, and the output
      // type is tested outside the loops.  (One read, one wait, one store at a time under a three-way branch took
      // 3.5 us per half -- for 16-bit output, half the bytes, even longer.)
      constexpr int NI = BN / 8, NB = (NI + 1) / 2;             // 16-byte reads per lane and half; per batch
      auto rows_out = [&](auto kind) {
        constexpr int KIND = decltype(kind)::value;
#pragma unroll
        for (int b0 = 0; b0 < NI; b0 += NB) {
          f32x4 v[NB];   // (a vector type: an array of structs would live in scratch memory)
#pragma unroll
          for (int u = 0; u < NB; ++u) {
            const int idx = (b0 + u) * 64 + lane;
            const int r = idx / (BN / 4), c4 = idx - r * (BN / 4);
            if (b0 + u < NI) v[u] = *(const f32x4*)(Tw + r * TS + 4 * c4);
          }
#pragma unroll
          for (int u = 0; u < NB; ++u) {
            const int idx = (b0 + u) * 64 + lane;
            const int r = idx / (BN / 4), c4 = idx - r * (BN / 4);
            const int m = mrow0 + r, n = n0 + 4 * c4;
            if (b0 + u < NI && m < M && n < out) {
              const long long o = (long long)m * out + n;
              if constexpr (KIND == BTC_F32) {
                *(f32x4*)((float*)Y + o) = v[u];
              } else if constexpr (KIND == BTC_BF16) {
                *(uint2*)((uint16_t*)Y + o) = make_uint2(bf16_bits(v[u].x) | (bf16_bits(v[u].y) << 16),
                                                         bf16_bits(v[u].z) | (bf16_bits(v[u].w) << 16));
              } else {
                *(uint2*)((uint16_t*)Y + o) = make_uint2(f16_bits(v[u].x) | (f16_bits(v[u].y) << 16),
                                                         f16_bits(v[u].z) | (f16_bits(v[u].w) << 16));
              }
            }
          }
        }
      };
      if (y_dtype == BTC_F32) rows_out(std::integral_constant<int, BTC_F32>{});
      else if (y_dtype == BTC_BF16) rows_out(std::integral_constant<int, BTC_BF16>{});
      else rows_out(std::integral_constant<int, BTC_F16>{});
    } else {
      for (int idx = lane; idx < 32 * BN; idx += 64) {
        const int r = idx / BN, cc = idx - r * BN;
        const int m = mrow0 + r, n = n0 + cc;
        if (m < M && n < out) {
          const float v = Tw[r * TS + cc];
          const long long o = (long long)m * out + n;
          if (y_dtype == BTC_F32) ((float*)Y)[o] = v;
          else if (y_dtype == BTC_BF16) ((__hip_bfloat16*)Y)[o] = __float2bfloat16(v);
          else ((__half*)Y)[o] = __float2half_rn(v);
        }
      }
    }
    wave_lds_sync();                                           // before the second half overwrites the rows
    if (wave == 0) WSTAMP(0, 4 + a);
  }
#ifdef BTC_WIDE_STAMPS
  __builtin_amdgcn_s_waitcnt(0x0F70);                          // the stores have left
  if (wave == 0) WSTAMP(0, 6);
#endif
}

static int pitch_of(const Dims& d) { return (d.in + kKT - 1) / kKT * kKT; }

// weight rows per workgroup / 32: the widest tile that still gives every compute unit work
static int pick_nf(const Dims& d, int M) {
  const int m_blocks = (M + kBM - 1) / kBM;
  int best = 5;
  double best_cost = 1e300;
  for (int nf = 3; nf <= 5; ++nf) {
    const long long tiles = (long long)m_blocks * ((d.out + 32 * nf - 1) / (32 * nf));
    const double cost = (double)((tiles + 255) / 256) * (0.3 + 0.155 * nf);   // rounds x time of a k-tile
    if (cost < best_cost - 1e-9) {
      best_cost = cost;
      best = nf;
    }
  }
  return best;
}

template <int NF, bool BF16>
static btc_status launch(hipStream_t q, const Dims& d, const unsigned char* WB, int pitch, const float* alpha,
                         const float* mu, const void* X, const float* rs, int M, void* Y, int y_dtype) {
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemm_wide_kernel<NF, BF16>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  const int m_blocks = (M + kBM - 1) / kBM, n_blocks = (d.out + 32 * NF - 1) / (32 * NF);
  // split of the eight XCDs over m blocks (gm) and n blocks (8 / gm): least bytes read by the chip,
  // gm x (weight bytes) + (8 / gm) x (activation bytes); no more XCD rows than m blocks
  int gm = 1;
  {
    const double wbytes = (double)d.out * pitch, abytes = (double)M * d.in * 2;
    double best = 1e300;
    for (int g = 1; g <= 8; g *= 2) {
      if (g > m_blocks && g > 1) break;
      if (8 / g > n_blocks && g < 8) continue;
      const double t = g * wbytes + (8 / g) * abytes;
      if (t < best) {
        best = t;
        gm = g;
      }
    }
  }
  const int grid = 8 * ((m_blocks + gm - 1) / gm) * ((n_blocks + 8 / gm - 1) / (8 / gm));
  gemm_wide_kernel<NF, BF16><<<grid, (kMW + kLW) * 64, 3 * kXB + 3 * kWBmax, q>>>(
      d.in, d.out, WB, pitch, alpha, mu, (const uint16_t*)X, rs, M, Y, y_dtype, m_blocks, n_blocks, gm);
  return launch_status();
}

}  // namespace wide

#ifdef BTC_WIDE_STAMPS
extern "C" int btc_debug_wide_stamps(unsigned long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(wide::g_stamps), sizeof(unsigned long long) * n);
}
#endif

bool gemm_wide_covers(const Dims& d, int M) {
  // worth its first kernel only when the 256 x 160 output tiles fill the chip (below that the tiled
  // kernel, which can split a call along k, is as fast or faster)
  if (M < 512 || d.b > 16) return false;
  if ((long long)((M + wide::kBM - 1) / wide::kBM) * ((d.out + 159) / 160) < 224) return false;
  if (d.in % 16 != 0) return false;                           // 16-byte pieces of an activation row
  if ((long long)M * d.in * 2 >= (1LL << 31)) return false;   // 32-bit buffer offsets
  if ((long long)d.out * wide::pitch_of(d) >= (1LL << 31)) return false;
  return true;
}

// the sign bytes, then the fp32 sums of the activation rows
static size_t sign_bytes(const Dims& d) { return ((size_t)d.out * wide::pitch_of(d) + 255) & ~(size_t)255; }
size_t gemm_wide_workspace_bytes(const Dims& d, int M) { return sign_bytes(d) + (((size_t)M * 4 + 255) & ~(size_t)255); }

btc_status gemm_wide(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                     const float* alpha, const float* mu, const void* X, int is_bf16, int M, void* Y, int y_dtype,
                     void* workspace, size_t workspace_bytes) {
  using namespace wide;
  if (!workspace || workspace_bytes < gemm_wide_workspace_bytes(d, M)) return BTC_ERR_WORKSPACE;
  const int pitch = pitch_of(d);
  unsigned char* WB = (unsigned char*)workspace;
  float* rs = (float*)(WB + sign_bytes(d));
  const long long pieces = (long long)d.out * (pitch / 16);
  // a few thousand blocks that each walk over the pieces (the table in LDS is filled once per block)
  int expand_blocks = (int)std::min<long long>((pieces + 255) / 256, 2048);
  const int sum_blocks = (M + 3) / 4;
  if (d.v == 10 && d.b <= 10 && d.wpr <= kRowWords)      // blocks walk over groups of kRowsAtOnce rows
    expand_blocks = std::min((d.out + kRowsAtOnce - 1) / kRowsAtOnce, 2048);
  if (is_bf16)
    expand_signs_kernel<true><<<expand_blocks + sum_blocks, 256, 0, q>>>(d, packed, codebook, WB, pitch, expand_blocks,
                                                                         (const uint16_t*)X, M, rs);
  else
    expand_signs_kernel<false><<<expand_blocks + sum_blocks, 256, 0, q>>>(d, packed, codebook, WB, pitch, expand_blocks,
                                                                          (const uint16_t*)X, M, rs);
  btc_status st = launch_status();
  if (st != BTC_OK) return st;
  const int nf = pick_nf(d, M);
#define BTC_WIDE_CASE(NFV)                                                                                  \
  if (nf == NFV)                                                                                            \
    return is_bf16 ? launch<NFV, true>(q, d, WB, pitch, alpha, mu, X, rs, M, Y, y_dtype)                        \
                   : launch<NFV, false>(q, d, WB, pitch, alpha, mu, X, rs, M, Y, y_dtype)
  BTC_WIDE_CASE(3);
  BTC_WIDE_CASE(4);
  BTC_WIDE_CASE(5);
#undef BTC_WIDE_CASE
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace btc
