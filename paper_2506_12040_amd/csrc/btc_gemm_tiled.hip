// Tuned prefill product for chunk length 10:  Y[M][out] = X[M][in] . W_hat^T.
//
// At many activation rows the layer is a dense contraction, so the index
// tiles are decoded into +-1 tiles in LDS (exact in bf16 and fp16) and
// contracted on the matrix cores with fp32 accumulation; alpha and mu are
// applied afterwards in fp32 (Algorithm "Binary Transformation and
// Compression": W_hat = alpha * B_hat + mu).
//
// Roles inside a workgroup (wave specialisation):
//   * 4 contraction waves, stacked along M.  Wave w owns 64 activation rows
//     and all BN = 32 NF weight rows of the workgroup: 2 x NF accumulators
//     of MFMA 32x32x16.  Both operands come from LDS and nothing else: two
//     16-byte reads (activations) and NF 8-byte reads (weights) per k-slice
//     of 16, issued one slice ahead of the MFMAs that use them.  The loop of
//     these waves holds no global load, so the in-order issue of the one
//     contraction wave per SIMD never waits for memory.
//   * 4 staging waves.  They copy the next k-tile of the activation block
//     (256 rows x 80 columns; coalesced 16-byte loads, ten lanes per row,
//     requested two tiles ahead) into LDS, and decode the next k-tile of the
//     weights: a work item turns 4 chunk indices of one weight row into 40
//     bytes, one byte per weight -- the HIGH byte of +-1.0 in the operand's
//     format.  A contraction wave widens 8 such bytes to an MFMA operand
//     with four byte permutes.  One byte per weight halves the LDS space and
//     traffic of the weight tile, which is what lets the whole activation
//     tile live in LDS next to it.
//   * one barrier per k-tile of 80 columns (8 chunks), two tile buffers.  A
//     contraction wave reaches the barrier with the operands of the tile's
//     last k-slice already in registers, reads the first slice of the next
//     tile right after it and only then issues the last slice's MFMAs.
//
// Workgroups are numbered so that all workgroups of one block of activation
// rows land on the same XCD: its 4 MB L2 then keeps that block of X resident
// while the weight-row blocks stream through.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <type_traits>

#include "btc_internal.h"

namespace btc {
namespace tiled {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kV = 10;                  // chunk length this kernel is built for
constexpr int kCH = 8;                  // chunks per k-tile
constexpr int kKT = kV * kCH;           // 80 columns per k-tile = 5 k-slices of 16
constexpr int kNS = kKT / 16;           // k-slices per tile
constexpr int kXRS = 2 * kKT + 16;      // bytes per staged activation row: an odd multiple of 16
constexpr int kWRS = kKT + 8;           // bytes per decoded weight row: an odd multiple of 8
constexpr int kBM = 256;                // activation rows per workgroup
constexpr int kXT = kBM * kXRS;         // bytes of one activation tile buffer
constexpr int kMW = 4;                  // contraction waves
constexpr int kDW = 4;                  // staging waves (8 waves per workgroup: 2 per SIMD, 256 registers each)
constexpr int kXL = 11;                 // activation loads per staging thread and tile (the last one partial)
constexpr int kRsrcFlags = 0x00020000;

template <bool BF16>
__device__ __forceinline__ f32x16 mfma32(const uint4& a, const uint4& b, const f32x16& c) {
  if constexpr (BF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

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
__device__ __forceinline__ uint4 widen_weights(const uint2& raw, uint32_t low) {
  uint4 r;
  r.x = __builtin_amdgcn_perm(raw.x, low, 0x05000400u);
  r.y = __builtin_amdgcn_perm(raw.x, low, 0x07000600u);
  r.z = __builtin_amdgcn_perm(raw.y, low, 0x05000400u);
  r.w = __builtin_amdgcn_perm(raw.y, low, 0x07000600u);
  return r;
}

template <int NF, bool BF16>
__global__ __launch_bounds__((kMW + kDW) * 64) void gemm_tiled_kernel(
    Dims d, const uint32_t* __restrict__ packed, const uint32_t* __restrict__ codebook,
    const float* __restrict__ alpha, const float* __restrict__ mu, const uint16_t* __restrict__ X, int M,
    void* __restrict__ Y, int y_dtype, int m_blocks, int n_blocks, int tiles_per_split, float* __restrict__ part,
    float* __restrict__ rpart) {
  constexpr int BN = 32 * NF;
  constexpr int kWT = BN * kWRS;                         // bytes of one weight tile buffer
  extern __shared__ __align__(16) unsigned char smem[];
  // LDS: activation tiles [2][256][kXRS] at 0, weight tiles [2][BN][kWRS], codeword table [2^b][32 bytes]
  unsigned char* const WT = smem + 2 * kXT;
  unsigned char* const E = WT + 2 * kWT;

  // ---- workgroup -> (m block, n block); consecutive ids go to consecutive XCDs
  int mb, nb, sp;                                       // activation-row block, weight-row block, k split
  {
    const int per_split = m_blocks >= 8 ? 8 * ((m_blocks + 7) >> 3) * n_blocks : m_blocks * n_blocks;
    sp = blockIdx.x / per_split;
    const int L = blockIdx.x - sp * per_split;
    if (m_blocks >= 8) {
      const int xcd = L & 7, s = L >> 3;
      const int per_xcd = (m_blocks + 7) >> 3;
      mb = xcd + 8 * (s % per_xcd);
      nb = s / per_xcd;
    } else {
      mb = L % m_blocks;
      nb = L / m_blocks;
    }
    if (mb >= m_blocks || nb >= n_blocks) return;
  }
  const int m0 = mb * kBM, n0 = nb * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ntiles = (d.nchunks + kCH - 1) / kCH;
  // this workgroup's share of the k-tiles (the host makes every split non-empty)
  const int t_begin = sp * tiles_per_split;
  const int nt = min(ntiles, t_begin + tiles_per_split) - t_begin;
  const int k_lim = min(d.in, (t_begin + nt) * kKT);     // columns of this workgroup's share end here

  // Codeword table, built by all threads after each role has put its first global loads in
  // flight (the table needs a round trip of its own for the codebook).  An entry holds the ten
  // weight bytes of a codeword twice: at byte 0 for a chunk that starts on a dword of its row
  // (even position in its pair), and at byte 18 (i.e. shifted by two bytes in the second
  // 16-byte half) for the chunk behind it, so that a pair of chunks is put together from
  // whole dwords: {e0, e1, e2 | o0, o1, o2}.
  auto build_table = [&]() {
    const uint32_t hi = BF16 ? 0x3Fu : 0x3Cu;
    for (int k = tid; k < (1 << d.b); k += (kMW + kDW) * 64) {
      const uint32_t npat = ~codebook[k];
      uint32_t by[10];
#pragma unroll
      for (int t = 0; t < 10; ++t) by[t] = hi | (((npat >> t) & 1u) << 7);
      uint4 ev, od;
      ev.x = by[0] | (by[1] << 8) | (by[2] << 16) | (by[3] << 24);
      ev.y = by[4] | (by[5] << 8) | (by[6] << 16) | (by[7] << 24);
      ev.z = by[8] | (by[9] << 8);
      ev.w = 0u;
      od.x = (by[0] << 16) | (by[1] << 24);
      od.y = by[2] | (by[3] << 8) | (by[4] << 16) | (by[5] << 24);
      od.z = by[6] | (by[7] << 8) | (by[8] << 16) | (by[9] << 24);
      od.w = 0u;
      *(uint4*)(E + 32 * k) = ev;
      *(uint4*)(E + 32 * k + 16) = od;
    }
    __syncthreads();
  };

  if (wave >= kMW) {
    // =============================== staging waves ===============================
    // No branch below depends on the lane (threads without work of their own repeat a
    // neighbour's, writing the same values to the same place), and every stage issues the same
    // loads (those beyond the share return zeros): the number of loads in flight is a
    // compile-time fact, so a stage waits for its own tile only, not for the younger requests.
    const int did = tid - kMW * 64;                      // 0 .. 255
    // ---- activations: thread (row0, piece) copies piece `piece` (16 bytes) of the rows
    // row0 + 25 i of the tile, i = 0..10 (the last round covers rows 250..255 only)
    const __amdgpu_buffer_rsrc_t rX =
        __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, (int)((long long)M * d.in * 2), kRsrcFlags);
    const int xt = min(did, 249);
    const int xrow0 = xt / 10, xpiece = xt - 10 * xrow0;
    // Rows m >= M need no test of their own: X is row-major, so they lie past the end of the
    // buffer and the hardware range check returns zeros for them.
    uint32_t xv[kXL];                                    // byte offset of this thread's piece in round i, tile 0
    uint32_t xl[kXL];                                    // and where it goes in a tile buffer
#pragma unroll
    for (int i = 0; i < kXL; ++i) {
      const int row = min(xrow0 + 25 * i, kBM - 1);
      xv[i] = (uint32_t)(((long long)(m0 + row) * d.in + 8 * xpiece) * 2);
      xl[i] = (uint32_t)(row * kXRS + xpiece * 16);
    }
    uint4 XS[3][kXL];                                    // three tiles in flight
    auto load_x = [&](uint4 (&dst)[kXL], int t) {
      if ((t + 1) * kKT <= k_lim) {                      // the whole tile lies inside the share: scalar column offset
#pragma unroll
        for (int i = 0; i < kXL; ++i)
          dst[i] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rX, xv[i], t * kKT * 2, 0));
      } else {
        // `in` is a multiple of 16 for this kernel, so a piece lies wholly inside or outside the
        // row (or this workgroup's share of it); outside, bit 31 of the offset is set
        const uint32_t past = (uint32_t)(t * kKT + 8 * xpiece + 8 > k_lim) << 31;
#pragma unroll
        for (int i = 0; i < kXL; ++i)
          dst[i] = __builtin_bit_cast(
              uint4, __builtin_amdgcn_raw_buffer_load_b128(rX, (xv[i] + (uint32_t)(t * kKT) * 2u) | past, 0, 0));
      }
    };
    auto store_x = [&](const uint4 (&src)[kXL], int buf) {
#pragma unroll
      for (int i = 0; i < kXL; ++i) *(uint4*)(smem + buf * kXT + xl[i]) = src[i];
    };
    // ---- weights: a thread owns 4 chunks (a half of the 8 chunks a row has in a tile) of one of the
    // first 128 weight rows, and -- with 160 rows per workgroup -- threads 0..127 also own 2 chunks (a
    // quarter) of one of the rows 128..159.  The b-bit fields of either lie inside two words of
    // the row for every b <= 10, since they start at a multiple of 2 b bits.
    constexpr bool kQ = BN > 128;
    const uint32_t pk_bytes = (uint32_t)d.out * (uint32_t)d.wpr * 4u;
    const __amdgpu_buffer_rsrc_t rP = __builtin_amdgcn_make_buffer_rsrc((void*)packed, 0, (int)pk_bytes, kRsrcFlags);
    const bool has_h = (did & ~63) < 2 * min(BN, 128);   // wave-uniform
    const bool has_q = kQ && did < 128;                  // wave-uniform
    const int hr = min(did >> 1, BN - 1), hh = did & 1;
    const int qr = 128 + ((did & 127) >> 2), qq = did & 3;
    // rows past the end of the matrix start past the end of the buffer: zeros, i.e. index 0
    const uint32_t h_row = (uint32_t)(n0 + hr) * (uint32_t)d.wpr * 4u, h_bit = (uint32_t)(hh * 4 * d.b);
    const uint32_t q_row = (uint32_t)(n0 + qr) * (uint32_t)d.wpr * 4u, q_bit = (uint32_t)(qq * 2 * d.b);
    unsigned char* const h_dst = WT + hr * kWRS + hh * 40;
    unsigned char* const q_dst = WT + qr * kWRS + qq * 20;
    uint32_t IW[3][4];                                   // index words (half item: 0, 1; quarter item: 2, 3), three tiles in flight
    auto fetch = [&](uint32_t (&dst)[4], int t) {
      const uint32_t tb = (uint32_t)(t * kCH * d.b);
      if (has_h) {
        const uint32_t off = h_row + (((tb + h_bit) >> 5) << 2);
        dst[0] = __builtin_amdgcn_raw_buffer_load_b32(rP, off, 0, 0);
        dst[1] = __builtin_amdgcn_raw_buffer_load_b32(rP, off + 4u, 0, 0);
      }
      if (has_q) {
        const uint32_t off = q_row + (((tb + q_bit) >> 5) << 2);
        dst[2] = __builtin_amdgcn_raw_buffer_load_b32(rP, off, 0, 0);
        dst[3] = __builtin_amdgcn_raw_buffer_load_b32(rP, off + 4u, 0, 0);
      }
    };
    const uint32_t mask = (1u << d.b) - 1u;
    auto decode = [&](const uint32_t (&src)[4], int t, int buf) {
      const uint32_t tb = (uint32_t)(t * kCH * d.b);
      uint4 e[4], f[2];
      if (has_h) {
        const uint32_t sh = (tb + h_bit) & 31u;
        const uint32_t lo = __builtin_amdgcn_alignbit(src[1], src[0], sh);
        const uint32_t hi = src[1] >> sh;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const uint32_t code = __builtin_amdgcn_alignbit(hi, lo, (uint32_t)(c * d.b)) & mask;
          e[c] = *(const uint4*)(E + 32 * code + 16 * (c & 1));
        }
      }
      if (has_q) {
        const uint32_t sh = (tb + q_bit) & 31u;
        const uint32_t lo = __builtin_amdgcn_alignbit(src[3], src[2], sh);
        f[0] = *(const uint4*)(E + 32 * (lo & mask));
        f[1] = *(const uint4*)(E + 32 * ((lo >> d.b) & mask) + 16);
      }
      if (has_h) {
        uint2* dst = (uint2*)(h_dst + buf * kWT);
        dst[0] = make_uint2(e[0].x, e[0].y);
        dst[1] = make_uint2(e[0].z | e[1].x, e[1].y);
        dst[2] = make_uint2(e[1].z, e[2].x);
        dst[3] = make_uint2(e[2].y, e[2].z | e[3].x);
        dst[4] = make_uint2(e[3].y, e[3].z);
      }
      if (has_q) {
        uint32_t* dst = (uint32_t*)(q_dst + buf * kWT);
        dst[0] = f[0].x;
        dst[1] = f[0].y;
        dst[2] = f[0].z | f[1].x;
        dst[3] = f[1].y;
        dst[4] = f[1].z;
      }
    };
#pragma unroll
    for (int g = 0; g < 3; ++g) {                        // (beyond the share: out-of-range offsets, zeros)
      fetch(IW[g], t_begin + g);
      load_x(XS[g], t_begin + g);
    }
    build_table();
    // Tile lt goes to tile buffer lt % 2 between the barrier that ends tile lt - 2 and the one
    // that starts tile lt; its loads were requested three tiles earlier into register set lt % 3.
    auto stage = [&](int lt, auto variant) {
      constexpr int P2 = decltype(variant)::value % 2, P3 = decltype(variant)::value % 3;
      store_x(XS[P3], P2);
      decode(IW[P3], t_begin + lt, P2);
      fetch(IW[P3], t_begin + lt + 3);
      load_x(XS[P3], t_begin + lt + 3);
      __syncthreads();
    };
    // nt + 1 barriers in all; the last stage writes a tile that nobody reads into the buffers
    // whose tile (nt - 2) has been consumed
    for (int lt = 0;; lt += 6) {
      stage(lt, std::integral_constant<int, 0>{});
      if (lt + 1 > nt) break;
      stage(lt + 1, std::integral_constant<int, 1>{});
      if (lt + 2 > nt) break;
      stage(lt + 2, std::integral_constant<int, 2>{});
      if (lt + 3 > nt) break;
      stage(lt + 3, std::integral_constant<int, 3>{});
      if (lt + 4 > nt) break;
      stage(lt + 4, std::integral_constant<int, 4>{});
      if (lt + 5 > nt) break;
      stage(lt + 5, std::integral_constant<int, 5>{});
      if (lt + 6 > nt) break;
    }
    return;
  }

  // ================================= contraction waves =================================
  if (m0 + wave * 64 >= M) {                             // no activation rows for this wave: keep the barriers only
    build_table();
    __syncthreads();
    for (int lt = 0; lt < nt; ++lt) __syncthreads();
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

  // Operand addresses: lane (l32, h) holds elements 8 h .. 8 h + 7 of a k-slice of 16, of
  // activation row l32 of a fragment (A) and of weight row l32 of a block of 32 (B).
  const unsigned char* const a_lane = smem + (wave * 64 + l32) * kXRS + h * 16;
  const unsigned char* const b_lane = WT + l32 * kWRS + h * 8;
  const uint32_t low = BF16 ? 0x80u : 0x00u;
  uint4 afr[2][2];                                       // [register set][fragment]
  uint2 bfr[2][NF];                                      // [register set][weight block]
  float rsum[2] = {0.f, 0.f};                            // rows l32 and 32 + l32, this lane's half of the columns
  auto read_slice = [&](int set, int buf, int s) {
#pragma unroll
    for (int a = 0; a < 2; ++a) afr[set][a] = *(const uint4*)(a_lane + buf * kXT + a * 32 * kXRS + s * 32);
#pragma unroll
    for (int c = 0; c < NF; ++c) bfr[set][c] = *(const uint2*)(b_lane + buf * kWT + c * 32 * kWRS + s * 16);
  };
  build_table();
  __syncthreads();                                       // tile 0 staged
  read_slice(0, 0, 0);
  // A tile body: 5 k-slices; register sets alternate per slice, and since a tile has an odd
  // number of slices the set of its first slice follows the tile's parity, like its buffer.
  uint4 bw[2];                                           // widened weights, two sets in turn
  auto tile = [&](bool has_next, auto parity) {
    constexpr int P = decltype(parity)::value;
#pragma unroll
    for (int s = 0; s < kNS; ++s) {
      const int set = (P + s) & 1;
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < kNS) {
        read_slice(set ^ 1, P, s + 1);
      } else {
        __syncthreads();                                 // this tile is in registers; the next one is staged
        if (has_next) read_slice(set ^ 1, P ^ 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (s == 0) bw[0] = widen_weights(bfr[set][0], low);
#pragma unroll
      for (int c = 0; c < NF; ++c) {
        // order pinned: the permutes for the next block and the row-sum steps are issued in the
        // shadow of this block's two MFMAs and write registers no MFMA in flight reads
        __builtin_amdgcn_sched_barrier(0);
        const int g = s * NF + c;                        // blocks alternate between the two widened sets
        acc[0][c] = mfma32<BF16>(afr[set][0], bw[g & 1], acc[0][c]);
        __builtin_amdgcn_sched_barrier(0);
        if (c + 1 < NF) bw[(g + 1) & 1] = widen_weights(bfr[set][c + 1], low);
        else if (s + 1 < kNS) bw[(g + 1) & 1] = widen_weights(bfr[set ^ 1][0], low);
        __builtin_amdgcn_sched_barrier(0);
        acc[1][c] = mfma32<BF16>(afr[set][1], bw[g & 1], acc[1][c]);
        __builtin_amdgcn_sched_barrier(0);
        if (c < 4) {
          const uint32_t w0 = c == 0 ? afr[set][0].x : c == 1 ? afr[set][0].y : c == 2 ? afr[set][0].z : afr[set][0].w;
          const uint32_t w1 = c == 0 ? afr[set][1].x : c == 1 ? afr[set][1].y : c == 2 ? afr[set][1].z : afr[set][1].w;
          rsum[0] = pair_sum<BF16>(w0, rsum[0]);
          rsum[1] = pair_sum<BF16>(w1, rsum[1]);
        }
      }
      if (NF < 4) {                                      // the row-sum steps that found no block to hide behind
#pragma unroll
        for (int c = NF; c < 4; ++c) {
          const uint32_t w0 = c == 2 ? afr[set][0].z : afr[set][0].w;
          const uint32_t w1 = c == 2 ? afr[set][1].z : afr[set][1].w;
          rsum[0] = pair_sum<BF16>(w0, rsum[0]);
          rsum[1] = pair_sum<BF16>(w1, rsum[1]);
        }
      }
    }
  };
  for (int lt = 0; lt < nt; lt += 2) {
    tile(lt + 1 < nt, std::integral_constant<int, 0>{});
    if (lt + 1 < nt) tile(lt + 2 < nt, std::integral_constant<int, 1>{});
  }

  // ---- epilogue.  After the last barrier the tile buffers are free; each wave uses a part of
  // them to turn its accumulators (lane = weight row n, 16 activation rows per register set)
  // into rows of Y, so that a lane stores 4 consecutive outputs at once.
  constexpr int TS = BN + 4;                                   // floats per staged row
  float* Tw = (float*)smem + wave * (32 * TS);                 // 32 rows x BN of this wave
  float* rsb = (float*)smem + kMW * (32 * TS) + wave * 64;     // its 64 row sums
  // With a k split the workgroup leaves its raw sums and its share of the activation row sums
  // (one copy per weight-row block) in the workspace; a second kernel adds the splits
  // and applies alpha and mu.
  const bool split = part != nullptr;
  if (split) {
    Y = part + (size_t)sp * M * d.out;
    y_dtype = BTC_F32;
  }
  float al[NF], mn[NF];
#pragma unroll
  for (int c = 0; c < NF; ++c) {
    const int n = n0 + c * 32 + l32;
    al[c] = split ? 1.f : (n < d.out ? alpha[n] : 0.f);
    mn[c] = split ? 0.f : (n < d.out ? mu[n] : 0.f);
  }
  // row sums: the two lanes that shared a row add up, then every lane picks up the 32 sums it needs
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    rsum[a] += __shfl_xor(rsum[a], 32, 64);
    if (h == 0) {
      rsb[32 * a + l32] = rsum[a];
      const int m = m0 + wave * 64 + 32 * a + l32;
      if (split && m < M) rpart[((size_t)sp * n_blocks + nb) * M + m] = rsum[a];
    }
  }
  wave_lds_sync();
  const bool vec = (d.out & 3) == 0;                           // 4 outputs of a row are aligned and inside
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int mrow0 = m0 + wave * 64 + a * 32;
    float rs[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 v = *(const float4*)(rsb + a * 32 + 8 * g + 4 * h);
      rs[4 * g + 0] = v.x; rs[4 * g + 1] = v.y; rs[4 * g + 2] = v.z; rs[4 * g + 3] = v.w;
    }
    if (vec) {
#pragma unroll
      for (int c = 0; c < NF; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          Tw[(8 * (e >> 2) + 4 * h + (e & 3)) * TS + c * 32 + l32] = al[c] * acc[a][c][e] + mn[c] * rs[e];
      wave_lds_sync();
#pragma unroll 4
      for (int i = 0; i < BN / 8; ++i) {
        const int idx = i * 64 + lane;
        const int r = idx / (BN / 4), c4 = idx - r * (BN / 4);
        const float4 v = *(const float4*)(Tw + r * TS + 4 * c4);
        const int m = mrow0 + r, n = n0 + 4 * c4;
        if (m < M && n < d.out) {
          const long long o = (long long)m * d.out + n;
          if (y_dtype == BTC_F32) {
            *(float4*)((float*)Y + o) = v;
          } else if (y_dtype == BTC_BF16) {
            *(uint2*)((uint16_t*)Y + o) = make_uint2(bf16_bits(v.x) | (bf16_bits(v.y) << 16),
                                                     bf16_bits(v.z) | (bf16_bits(v.w) << 16));
          } else {
            *(uint2*)((uint16_t*)Y + o) = make_uint2(f16_bits(v.x) | (f16_bits(v.y) << 16),
                                                     f16_bits(v.z) | (f16_bits(v.w) << 16));
          }
        }
      }
      wave_lds_sync();                                         // before the second half overwrites the rows
    } else {
#pragma unroll
      for (int c = 0; c < NF; ++c) {
        const int n = n0 + c * 32 + l32;
        if (n >= d.out) continue;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int m = mrow0 + 8 * (e >> 2) + 4 * h + (e & 3);
          if (m >= M) continue;
          const float r = al[c] * acc[a][c][e] + mn[c] * rs[e];
          const long long o = (long long)m * d.out + n;
          if (y_dtype == BTC_F32) ((float*)Y)[o] = r;
          else if (y_dtype == BTC_BF16) ((__hip_bfloat16*)Y)[o] = __float2bfloat16(r);
          else ((__half*)Y)[o] = __float2half_rn(r);
        }
      }
    }
  }
}

template <int NF>
static size_t lds_bytes(int b) { return (size_t)2 * kXT + (size_t)2 * 32 * NF * kWRS + ((size_t)32 << b); }

// Second pass of a k-split call:  Y = alpha * (sum of the splits' raw sums) + mu * (sum of their
// activation row sums), in split order.  One small workgroup per (weight-row block, activation
// row): it is the only reader of that block's partial sums and of that block's copy of the row
// sums, so with `clear` it can hand the workspace back zero-filled (the decode entry point
// promises that to its callers) without a race.
__global__ __launch_bounds__(64) void split_reduce_kernel(float* __restrict__ part, float* __restrict__ rpart,
                                                          const float* __restrict__ alpha,
                                                          const float* __restrict__ mu, int M, int out, int bn,
                                                          int splits, void* __restrict__ Y, int y_dtype, int clear) {
  const int nb = blockIdx.x, m = blockIdx.y, tid = threadIdx.x;
  const int n_blocks = gridDim.x;
  const size_t total = (size_t)M * out;
  float rs = 0.f;
  for (int sp = 0; sp < splits; ++sp) rs += rpart[((size_t)sp * n_blocks + nb) * M + m];
  const size_t row = (size_t)m * out;
  const int n_begin = nb * bn, n_end = min(out, n_begin + bn);
  if ((out & 3) == 0) {
    for (int n = n_begin + 4 * tid; n < n_end; n += 4 * 64) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int sp = 0; sp < splits; ++sp) {
        float4* p = (float4*)(part + (size_t)sp * total + row + n);
        const float4 t = *p;
        v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
        if (clear) *p = make_float4(0.f, 0.f, 0.f, 0.f);
      }
      const float4 al = *(const float4*)(alpha + n), mn = *(const float4*)(mu + n);
      const float r0 = al.x * v.x + mn.x * rs, r1 = al.y * v.y + mn.y * rs, r2 = al.z * v.z + mn.z * rs,
                  r3 = al.w * v.w + mn.w * rs;
      if (y_dtype == BTC_F32) {
        *(float4*)((float*)Y + row + n) = make_float4(r0, r1, r2, r3);
      } else if (y_dtype == BTC_BF16) {
        *(uint2*)((uint16_t*)Y + row + n) =
            make_uint2(bf16_bits(r0) | (bf16_bits(r1) << 16), bf16_bits(r2) | (bf16_bits(r3) << 16));
      } else {
        *(uint2*)((uint16_t*)Y + row + n) =
            make_uint2(f16_bits(r0) | (f16_bits(r1) << 16), f16_bits(r2) | (f16_bits(r3) << 16));
      }
    }
  } else {
    for (int n = n_begin + tid; n < n_end; n += 64) {
      float v = 0.f;
      for (int sp = 0; sp < splits; ++sp) {
        float* p = part + (size_t)sp * total + row + n;
        v += *p;
        if (clear) *p = 0.f;
      }
      const float r = alpha[n] * v + mu[n] * rs;
      if (y_dtype == BTC_F32) ((float*)Y)[row + n] = r;
      else if (y_dtype == BTC_BF16) ((__hip_bfloat16*)Y)[row + n] = __float2bfloat16(r);
      else ((__half*)Y)[row + n] = __float2half_rn(r);
    }
  }
  if (clear) {
    __syncthreads();   // every thread has read the row sum
    if (tid < splits) rpart[((size_t)tid * n_blocks + nb) * M + m] = 0.f;
  }
}

struct Plan {
  int nf;               // weight rows per workgroup / 32
  int splits;           // workgroups that share one output tile along k
  int tiles_per_split;
  double est_us;        // modelled duration of the call
};

// Tile width and k split.  A workgroup occupies a compute unit, so the kernel lasts about
//   rounds x (k-tiles per workgroup) x (time per k-tile) + a fixed part,
// all fitted to measurements (microseconds): a k-tile of 80 columns costs half of 0.15 + 0.17 NF +
// 0.45 per contraction wave that has activation rows (the NF term is the decode and the weight
// operands, the wave term the activation tile: LDS time bounds the kernel); prologue and epilogue
// cost 10 + 2 NF.  Wide tiles win
// unless they leave compute units idle; then the k-tiles of an output tile are dealt to several
// workgroups, which costs a second pass over the partial sums.
static Plan make_plan(const Dims& d, int M) {
  const int m_blocks = (M + kBM - 1) / kBM;
  const int ntiles = (d.nchunks + kCH - 1) / kCH;
  const int waves = (min(M, kBM) + 63) / 64;
  Plan best{5, 1, ntiles, 0.0};
  double best_cost = 1e300;
  for (int nf = 2; nf <= 5; ++nf) {
    const double t_tile = 0.5 * (0.15 + 0.17 * nf + 0.45 * waves);
    const long long tiles_out = (long long)m_blocks * ((d.out + 32 * nf - 1) / (32 * nf));
    for (int sp = 1; sp <= 8; ++sp) {
      const int tps = (ntiles + sp - 1) / sp;
      if (sp > 1 && (tps < 8 || (sp - 1) * tps >= ntiles || M > 65535)) continue;   // short or empty splits; grid limit of the second pass
      const long long rounds = (tiles_out * sp + 255) / 256;
      double cost = (double)rounds * tps * t_tile + 10.0 + 2.0 * nf;
      if (sp > 1) cost += 2.0 + (double)sp * M * d.out * 4.0 / 3.0e6;   // second pass over the partials
      if (cost < best_cost) {
        best_cost = cost;
        best = Plan{nf, sp, tps, cost};
      }
    }
  }
  return best;
}

template <int NF, bool BF16>
static btc_status launch(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                         const float* alpha, const float* mu, const void* X, int M, void* Y, int y_dtype,
                         const Plan& plan, void* workspace, int clear_workspace) {
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemm_tiled_kernel<NF, BF16>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  const int m_blocks = (M + kBM - 1) / kBM, n_blocks = (d.out + 32 * NF - 1) / (32 * NF);
  int grid;
  if (m_blocks >= 8) grid = 8 * ((m_blocks + 7) / 8) * n_blocks;
  else grid = m_blocks * n_blocks;
  float* part = nullptr;
  float* rpart = nullptr;
  if (plan.splits > 1) {
    part = (float*)workspace;
    rpart = part + (size_t)plan.splits * M * d.out;
  }
  gemm_tiled_kernel<NF, BF16><<<grid * plan.splits, (kMW + kDW) * 64, lds_bytes<NF>(d.b), q>>>(
      d, packed, codebook, alpha, mu, (const uint16_t*)X, M, Y, y_dtype, m_blocks, n_blocks, plan.tiles_per_split,
      part, rpart);
  btc_status st = launch_status();
  if (st != BTC_OK || plan.splits == 1) return st;
  split_reduce_kernel<<<dim3(n_blocks, M), 64, 0, q>>>(part, rpart, alpha, mu, M, d.out, 32 * NF, plan.splits, Y, y_dtype,
                                                      clear_workspace);
  return launch_status();
}

}  // namespace tiled

bool gemm_tiled_covers(const Dims& d, int M) {
  if (d.v != tiled::kV || d.b > 10) return false;
  if (d.in % 16 != 0) return false;                           // 16-byte aligned, whole 16-element A loads
  if ((long long)M * d.in * 2 >= (1LL << 31)) return false;   // 32-bit buffer offsets
  // the index stream is addressed with 32-bit byte offsets too, 0x80000000 being the out-of-range one
  if ((long long)d.out * d.wpr * 4 >= (1LL << 31)) return false;
  return M >= 1;
}

double gemm_tiled_estimate_us(const Dims& d, int M) { return tiled::make_plan(d, M).est_us; }

size_t gemm_tiled_workspace_bytes(const Dims& d, int M) {
  const tiled::Plan plan = tiled::make_plan(d, M);
  if (plan.splits == 1) return 0;
  const size_t n_blocks = (d.out + 32 * plan.nf - 1) / (32 * plan.nf);
  return (size_t)plan.splits * M * ((size_t)d.out + n_blocks) * sizeof(float);
}

btc_status gemm_tiled(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                      const float* alpha, const float* mu, const void* X, int is_bf16, int M, void* Y, int y_dtype,
                      void* workspace, size_t workspace_bytes, int clear_workspace) {
  using namespace tiled;
  const Plan plan = make_plan(d, M);
  if (plan.splits > 1 && (!workspace || workspace_bytes < gemm_tiled_workspace_bytes(d, M))) return BTC_ERR_WORKSPACE;
#define BTC_TILED_CASE(NFV)                                                                                         \
  if (plan.nf == NFV)                                                                                               \
    return is_bf16 ? launch<NFV, true>(q, d, packed, codebook, alpha, mu, X, M, Y, y_dtype, plan, workspace,       \
                                      clear_workspace)                                                          \
                   : launch<NFV, false>(q, d, packed, codebook, alpha, mu, X, M, Y, y_dtype, plan, workspace,      \
                                       clear_workspace)
  BTC_TILED_CASE(2);
  BTC_TILED_CASE(3);
  BTC_TILED_CASE(4);
  BTC_TILED_CASE(5);
#undef BTC_TILED_CASE
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace btc
