// Prefill product on 8-bit (or 4-bit) activation codes with the integer matrix cores (section "Activation
// Quantization on sub-bit LLMs", W0.8A8 / W0.8A4), for many activation rows:
//   Y[m][i] = step[m] * (alpha_i * sum_k B_hat[i][k] Q[m][k] + mu_i * sum_k Q[m][k]) + lo[m] * wsum[i]
// (the matrix cores multiply signed bytes: Q - 128 goes in, 128 * sum_k B_hat[i][k] is added back from wsum)
// Same two-kernel scheme as the 16-bit route for many rows (btc_gemm_wide.hip): the sign matrix is expanded
// once per call into one byte per weight -- here the int8 numbers +1 and -1, which ARE the matrix-core
// operand, nothing is widened -- and the contraction kernel streams tiles of it and of the codes into LDS
// with load-to-LDS instructions.  MFMA i32 32x32x32 on int8: exact integer sums, twice the rate and half
// the activation bytes of the 16-bit route.  k-tiles of 128 bytes (8 pieces of 16); piece p of row r sits
// at position p ^ ((r / 2) % 8), which makes the 16-byte operand reads of 16 consecutive rows hit 16
// different bank groups.  The first kernel also adds up the codes of every activation row.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <type_traits>

#include "btc_internal.h"

namespace btc {
namespace wide8 {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kKT = 128;                // columns (bytes) per k-tile
constexpr int kBM = 256;                // activation rows per workgroup
constexpr int kXB = kBM * kKT;          // bytes of an activation tile buffer
constexpr int kMW = 4, kLW = 4;         // contraction waves, loader waves
constexpr int kXJ = kXB / 1024 / kLW;   // activation loads per loader wave and tile (8)
constexpr uint32_t kOob = 0x80000000u;  // buffer offset that is always out of range
constexpr int kRsrcFlags = 0x00020000;

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

// ---- first kernel: the sign matrix as int8 (+1 = 0x01, -1 = 0xFF), WB[out][pitch] (pitch = 128 * number
// of k-tiles; zero past column `in`), one thread per 16 bytes
// at a time; the first blocks of the grid (all but `expand_blocks`) add up the codes of the activation
// rows instead, one wave per row (exact integers).
constexpr int kRowsAtOnce = 4;      // rows of index words a block of the first kernel holds in LDS
constexpr int kRowWords = 1024;     // words per such row at most (longer rows: read from memory)

__global__ __launch_bounds__(256) void expand_signs_i8_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                              const uint32_t* __restrict__ codebook,
                                                              unsigned char* __restrict__ WB, int pitch, int expand_blocks,
                                                              const uint8_t* __restrict__ Q, int M, float* __restrict__ qs) {
  const int sum_blocks = (int)gridDim.x - expand_blocks;
  if ((int)blockIdx.x < sum_blocks) {
    const int m = (int)blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (m >= M) return;
    const uint4* row = (const uint4*)(Q + (size_t)m * d.in);             // `in` is a multiple of 16 here
    const int n16 = d.in / 16;
    uint32_t acc = 0u;
    for (int base = 0; base < n16; base += 64 * 8) {     // eight loads in flight per lane
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + 64 * u + lane;
        v[u] = i < n16 ? row[i] : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        acc = __builtin_amdgcn_udot4(v[u].x, 0x01010101u, acc, false);
        acc = __builtin_amdgcn_udot4(v[u].y, 0x01010101u, acc, false);
        acc = __builtin_amdgcn_udot4(v[u].z, 0x01010101u, acc, false);
        acc = __builtin_amdgcn_udot4(v[u].w, 0x01010101u, acc, false);
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) qs[m] = (float)acc;
    return;
  }
  const int pieces = pitch >> 4;
  const uint32_t id = (blockIdx.x - (uint32_t)sum_blocks) * 256u + threadIdx.x;       // out * pitch < 2^31
  const uint32_t mask = (1u << d.b) - 1u;
  if (d.v == 10 && d.b <= 10 && d.wpr <= kRowWords) {
    // Chunk length 10: the 16 columns of a piece lie inside three consecutive chunks.  Their
    // (inverted) patterns, from a table in LDS, are strung together, shifted to the piece's first
    // column, and every 4 bits are spread over the 4 bytes of a word by one 24-bit multiply.
    // A block takes kRowsAtOnce rows at a time: their index words are fetched once, coalesced, into
    // LDS, and the threads pick their three index fields from there.
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
        uint4 o = make_uint4(0u, 0u, 0u, 0u);
        if (pc * 16 < d.in) {                              // (`in` is a multiple of 16: a piece is wholly inside or outside)
          const uint32_t* prow = words + r * d.wpr;
          const int j0 = (pc * 16) / 10, t0 = pc * 16 - 10 * j0;
          uint32_t bits = 0u;
#pragma unroll
          for (int u = 0; u < 3; ++u) {
            const int j = j0 + u;
            if (j < d.nchunks) {
              const uint32_t bit = (uint32_t)j * (uint32_t)d.b;
              const uint32_t w0 = bit >> 5, sh = bit & 31u;
              const uint32_t lo = prow[w0];
              const uint32_t hi = prow[w0 + 1];            // (one word past the row at most: inside `words`, shifted out)
              bits |= npat[__builtin_amdgcn_alignbit(hi, lo, sh) & mask] << (10 * u);
            }
          }
          const uint32_t n16 = bits >> t0;
          uint32_t w[4];
#pragma unroll
          for (int q = 0; q < 4; ++q)   // +1 = 0x01, -1 = 0xFF = 0x01 ^ 0xFE
            w[q] = 0x01010101u ^ (((__umul24((n16 >> (4 * q)) & 0xFu, 0x204081u)) & 0x01010101u) * 0xFEu);
          o = make_uint4(w[0], w[1], w[2], w[3]);
        }
        *(uint4*)(WB + (size_t)(row0 + r) * pitch + (size_t)pc * 16) = o;
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
      uint4 o = make_uint4(0u, 0u, 0u, 0u);
      if (pc * 16 < d.in) {                              // (`in` is a multiple of 16: a piece is wholly inside or outside)
        const uint32_t* prow = packed + (size_t)row * d.wpr;
        const int j0 = (pc * 16) / 10, t0 = pc * 16 - 10 * j0;
        uint32_t bits = 0u;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
          const int j = j0 + u;
          if (j < d.nchunks) {
            const uint32_t bit = (uint32_t)j * (uint32_t)d.b;
            const uint32_t w0 = bit >> 5, sh = bit & 31u;
            const uint32_t lo = prow[w0];
            const uint32_t hi = (sh + d.b > 32u) ? prow[w0 + 1] : 0u;   // inside the row whenever the field crosses
            bits |= npat[__builtin_amdgcn_alignbit(hi, lo, sh) & mask] << (10 * u);
          }
        }
        const uint32_t n16 = bits >> t0;
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)   // +1 = 0x01, -1 = 0xFF = 0x01 ^ 0xFE
          w[q] = 0x01010101u ^ (((__umul24((n16 >> (4 * q)) & 0xFu, 0x204081u)) & 0x01010101u) * 0xFEu);
        o = make_uint4(w[0], w[1], w[2], w[3]);
      }
      *(uint4*)(WB + (size_t)row * pitch + (size_t)pc * 16) = o;
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
        pat = 0xFFFFFFFFu;
        if (j < d.nchunks) {
          const long long bit = (long long)j * d.b;
          const int w0 = (int)(bit >> 5), sh = (int)(bit & 31);
          const uint32_t lo = prow[w0];
          const uint32_t hi = (sh + d.b > 32) ? prow[w0 + 1] : 0u;   // inside the row whenever the field crosses
          pat = codebook[__builtin_amdgcn_alignbit(hi, lo, (uint32_t)sh) & mask];
        }
        have = true;
      }
      // columns past `in` are zero: they meet the code 0, which enters the matrix cores as -128
      const uint32_t byte = k + e < d.in ? (((pat >> t) & 1u) ? 0x01u : 0xFFu) : 0u;
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

// ---- second kernel: the contraction
template <int NF>
__global__ __launch_bounds__((kMW + kLW) * 64) void gemm_wide_i8_kernel(
    int in, int out, const unsigned char* __restrict__ WB, int pitch, const float* __restrict__ alpha,
    const float* __restrict__ mu, const float* __restrict__ wsum, const uint8_t* __restrict__ Q,
    const float* __restrict__ qs_all, const float* __restrict__ lo_all, const float* __restrict__ step_all, int M,
    void* __restrict__ Y, int y_dtype, int m_blocks, int n_blocks, int gm) {
  constexpr int BN = 32 * NF;
  constexpr int kWB = BN * kKT;                          // bytes of a weight tile buffer (whole 1 KB loads)
  constexpr int kWJ = kWB / 1024;                        // weight loads per tile
  extern __shared__ __align__(16) unsigned char smem[];
  // LDS: activation tiles [3][256 rows][128 bytes] at 0, then weight tiles [3][BN][128]
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
    const __amdgpu_buffer_rsrc_t rX = __builtin_amdgcn_make_buffer_rsrc((void*)Q, 0, (int)((long long)M * in), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rW =
        __builtin_amdgcn_make_buffer_rsrc((void*)WB, 0, (int)((long long)out * pitch), kRsrcFlags);
    // Load i of this wave fills positions 64 (kXJ lw + i) + lane of the activation tile (8 per row).  Rows
    // m >= M lie past the end of the buffer: the hardware range check makes the load store zeros.
    uint32_t xv[kXJ];                                    // byte offset of this lane's piece in tile 0
    int xp[kXJ];                                         // its piece number (for the ragged last tile)
#pragma unroll
    for (int i = 0; i < kXJ; ++i) {
      const int g = 64 * (kXJ * lw + i) + lane;
      const int row = g >> 3, pos = g & 7;
      xp[i] = pos ^ ((row >> 1) & 7);
      xv[i] = (uint32_t)((long long)(m0 + row) * in + 16 * xp[i]);
    }
    constexpr int kWI = (kWJ + kLW - 1) / kLW;
    uint32_t wv[kWI];
#pragma unroll
    for (int i = 0; i < kWI; ++i) {
      const int g = 64 * (lw + kLW * i) + lane;
      const int row = g >> 3, pos = g & 7;
      wv[i] = (lw + kLW * i < kWJ) ? (uint32_t)((long long)(n0 + row) * pitch + 16 * (pos ^ ((row >> 1) & 7))) : kOob;
    }
    auto issue = [&](int t, int buf) {
      if (t >= nt) return;                               // (uniform)
      unsigned char* const xb = smem + buf * kXB + kXJ * lw * 1024;
      if ((t + 1) * kKT <= in) {                         // the whole tile lies inside the rows: scalar column offset
#pragma unroll
        for (int i = 0; i < kXJ; ++i) load_to_lds_16(rX, xb + i * 1024, xv[i], t * kKT);
      } else {
        // `in` is a multiple of 16 for this kernel, so a piece lies wholly inside or outside the row
#pragma unroll
        for (int i = 0; i < kXJ; ++i) {
          const uint32_t off = (t * kKT + 16 * xp[i] + 16 > in) ? kOob : xv[i] + (uint32_t)(t * kKT);
          load_to_lds_16(rX, xb + i * 1024, off, 0);
        }
      }
#pragma unroll
      for (int i = 0; i < kWI; ++i)
        if (lw + kLW * i < kWJ)                          // (uniform)
          load_to_lds_16(rW, WT + buf * kWB + (lw + kLW * i) * 1024, wv[i], t * kKT);
    };
    // Tile t lives in buffer t % 3.  Its loads are issued right after the barrier that ends tile
    // t - 3 (whose buffer it takes over) and must have landed at the barrier that ends tile t - 1.
    issue(0, 0);
    issue(1, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)
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
  i32x16 acc[2][NF];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < NF; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][c][e] = 0;

  // Lane (l32, h) holds bytes 16 h .. 16 h + 15 of a k-step of 32, of activation row l32 of a fragment (A)
  // and of weight row l32 of a block (B): piece 2 s + h of the row, stored at that number ^ swz,
  // swz = (row / 2) % 8 -- the same for every row this lane reads (rows differ by multiples of 32).
  const int swz = (l32 >> 1) & 7;
  const uint32_t a_row = (uint32_t)((wave * 64 + l32) * kKT);
  const uint32_t b_row = (uint32_t)(3 * kXB + l32 * kKT);
  uint32_t p_off[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) p_off[s] = (uint32_t)(((2 * s + h) ^ swz) * 16);
  i32x4 afr[2][2];                                       // [register set][fragment]
  i32x4 bfr[2][NF];                                      // [register set][weight block]
  auto read_step = [&](int set, int xoff, int woff, int s) {
#pragma unroll
    for (int a = 0; a < 2; ++a) afr[set][a] = *(const i32x4*)(smem + (uint32_t)xoff + a_row + p_off[s] + a * 32 * kKT);
#pragma unroll
    for (int c = 0; c < NF; ++c) bfr[set][c] = *(const i32x4*)(smem + (uint32_t)woff + b_row + p_off[s] + c * 32 * kKT);
  };
  __syncthreads();                                       // tiles 0 and 1 are in LDS
  read_step(0, 0, 0, 0);
  // 4 k-steps per tile; the operands of step s + 1 are read while step s is contracted, those of the next
  // tile's first step right after the barrier that the last step starts with.
  auto tile = [&](int xoff, int woff, int xnext, int wnext, bool has_next) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int set = s & 1;
      __builtin_amdgcn_sched_barrier(0);
      if (s < 3) {
        read_step(set ^ 1, xoff, woff, s + 1);
      } else {
        __syncthreads();                                 // this tile is in registers; the next one is in LDS
        if (has_next) read_step(set ^ 1, xnext, wnext, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      // the matrix cores take SIGNED bytes: code - 128 (top bit flipped) goes in, and the epilogue adds
      // 128 * (sum of the row's signs) back
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int e = 0; e < 4; ++e) afr[set][a][e] ^= (int)0x80808080u;
#pragma unroll
      for (int c = 0; c < NF; ++c) {
        acc[0][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(afr[set][0], bfr[set][c], acc[0][c], 0, 0, 0);
        acc[1][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(afr[set][1], bfr[set][c], acc[1][c], 0, 0, 0);
      }
    }
  };
  {
    int b0 = 0;                                          // buffer of the current tile
    for (int t = 0; t < nt; ++t) {
      const int b1 = b0 == 2 ? 0 : b0 + 1;
      tile(b0 * kXB, b0 * kWB, b1 * kXB, b1 * kWB, t + 1 < nt);
      b0 = b1;
    }
  }

  // ---- epilogue.  After the last barrier the tile buffers are free; each wave uses a part of
  // them to turn its accumulators (lane = weight row n, 16 activation rows per register set)
  // into rows of Y, so that a lane stores 4 consecutive outputs at once.
  constexpr int TS = BN + 4;                                   // floats per staged row
  float* Tw = (float*)smem + wave * (32 * TS);                 // 32 rows x BN of this wave
  float* rowp = (float*)smem + kMW * (32 * TS) + wave * 192;   // per activation row: sum of codes, step, offset
  float al[NF], mn[NF], ws[NF], kc[NF];
#pragma unroll
  for (int c = 0; c < NF; ++c) {
    const int n = n0 + c * 32 + l32;
    al[c] = n < out ? alpha[n] : 0.f;
    mn[c] = n < out ? mu[n] : 0.f;
    ws[c] = n < out ? wsum[n] : 0.f;
    // alpha * 128 * (sum of the row's signs), from wsum = alpha * (sum of signs) + mu * in
    kc[c] = 128.0f * (ws[c] - mn[c] * (float)in);
  }
  {
    const int m = m0 + wave * 64 + lane;
    rowp[lane] = m < M ? qs_all[m] : 0.f;
    rowp[64 + lane] = m < M ? step_all[m] : 0.f;
    rowp[128 + lane] = m < M ? lo_all[m] : 0.f;
  }
  wave_lds_sync();
  const bool vec = (out & 3) == 0;                             // 4 outputs of a row are aligned and inside
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int mrow0 = m0 + wave * 64 + a * 32;
    float qs[16], st[16], lw[16];                              // of the 16 activation rows this lane's registers hold
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = a * 32 + 8 * g + 4 * h + e;
        qs[4 * g + e] = rowp[r];
        st[4 * g + e] = rowp[64 + r];
        lw[4 * g + e] = rowp[128 + r];
      }
    }
#pragma unroll
    for (int c = 0; c < NF; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e)
        Tw[(8 * (e >> 2) + 4 * h + (e & 3)) * TS + c * 32 + l32] = st[e] * (al[c] * (float)acc[a][c][e] + mn[c] * qs[e] + kc[c]) + lw[e] * ws[c];
    wave_lds_sync();
    if (vec) {
      // The staged rows leave in batches: all LDS reads of a batch are issued, then its stores, and the output
      // type is tested outside the loops (one read, one wait, one store at a time under a three-way branch took
      // 3.5 us per half).
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
  }
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

template <int NF>
static btc_status launch(hipStream_t q, const Dims& d, const unsigned char* WB, int pitch, const float* alpha,
                         const float* mu, const float* wsum, const uint8_t* Q, const float* qs, const float* lo,
                         const float* step, int M, void* Y, int y_dtype) {
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemm_wide_i8_kernel<NF>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  const int m_blocks = (M + kBM - 1) / kBM, n_blocks = (d.out + 32 * NF - 1) / (32 * NF);
  // split of the eight XCDs over m blocks (gm) and n blocks (8 / gm): least bytes read by the chip,
  // gm x (weight bytes) + (8 / gm) x (activation bytes); no more XCD rows than m blocks
  int gm = 1;
  {
    const double wbytes = (double)d.out * pitch, abytes = (double)M * d.in * 1;
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
  gemm_wide_i8_kernel<NF><<<grid, (kMW + kLW) * 64, 3 * kXB + 3 * 32 * NF * kKT, q>>>(
      d.in, d.out, WB, pitch, alpha, mu, wsum, Q, qs, lo, step, M, Y, y_dtype, m_blocks, n_blocks, gm);
  return launch_status();
}

// the sign bytes, then the fp32 sums of the code rows
static size_t sign_bytes(const Dims& d) { return ((size_t)d.out * pitch_of(d) + 255) & ~(size_t)255; }

}  // namespace wide8

bool gemm_wide_i8_covers(const Dims& d, int M) {
  // worth its first kernel only when the 256 x 160 output tiles fill the chip
  if (M < 512 || d.b > 16) return false;
  if ((long long)((M + wide8::kBM - 1) / wide8::kBM) * ((d.out + 159) / 160) < 224) return false;
  if (d.in % 16 != 0) return false;                           // 16-byte pieces of a code row
  if ((long long)M * d.in >= (1LL << 31)) return false;       // 32-bit buffer offsets
  if ((long long)d.out * wide8::pitch_of(d) >= (1LL << 31)) return false;
  return true;
}

size_t gemm_wide_i8_workspace_bytes(const Dims& d, int M) {
  return wide8::sign_bytes(d) + (((size_t)M * 4 + 255) & ~(size_t)255);
}

btc_status gemm_wide_i8(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                        const float* alpha, const float* mu, const float* wsum, const uint8_t* Q, const float* lo,
                        const float* step, int M, void* Y, int y_dtype, void* workspace, size_t workspace_bytes) {
  using namespace wide8;
  if (!workspace || workspace_bytes < gemm_wide_i8_workspace_bytes(d, M)) return BTC_ERR_WORKSPACE;
  const int pitch = pitch_of(d);
  unsigned char* WB = (unsigned char*)workspace;
  float* qs = (float*)(WB + sign_bytes(d));
  const long long pieces = (long long)d.out * (pitch / 16);
  // a few thousand blocks that each walk over the pieces
  int expand_blocks = (int)std::min<long long>((pieces + 255) / 256, 2048);
  const int sum_blocks = (M + 3) / 4;
  if (d.v == 10 && d.b <= 10 && d.wpr <= kRowWords)      // blocks walk over groups of kRowsAtOnce rows
    expand_blocks = std::min((d.out + kRowsAtOnce - 1) / kRowsAtOnce, 2048);
  expand_signs_i8_kernel<<<expand_blocks + sum_blocks, 256, 0, q>>>(d, packed, codebook, WB, pitch, expand_blocks, Q, M, qs);
  btc_status st = launch_status();
  if (st != BTC_OK) return st;
  const int nf = pick_nf(d, M);
  if (nf == 3) return launch<3>(q, d, WB, pitch, alpha, mu, wsum, Q, qs, lo, step, M, Y, y_dtype);
  if (nf == 4) return launch<4>(q, d, WB, pitch, alpha, mu, wsum, Q, qs, lo, step, M, Y, y_dtype);
  return launch<5>(q, d, WB, pitch, alpha, mu, wsum, Q, qs, lo, step, M, Y, y_dtype);
}

}  // namespace btc
