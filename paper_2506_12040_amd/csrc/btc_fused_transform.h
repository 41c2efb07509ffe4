// The online activation transform of ONE activation row, computed by a workgroup into LDS in front of a decode
// product (section "Learnable Transformation": T = D P, D a diagonal sign matrix, P = P1 (x) P2;
// "Integration into Transformer Architecture": X <- X T at inference):
//     x'[j1 n2 + j2] = sum_{i1, i2} sigma[i] x[i] P1[i1][j1] P2[i2][j2],     i = i1 n2 + i2
// Every workgroup of a decode kernel needs the whole transformed row, so every workgroup computes it: with the
// row reshaped to n1 x n2 that is  P1^T (sigma x) P2,  two small dense contractions (1.5 Mflop at 64 x 80,
// 6.5 Mflop at 108 x 128) on the matrix cores (MFMA 32x32x16 f16, fp32 accumulate):
//   stage 1:  D1[i1][j2] = sum_i2 (sigma x)[i1][i2] P2[i2][j2]    A = the row itself from global memory in operand
//             layout (16 bytes per lane, signs applied in registers: exact); B = P2, prepared
//   stage 2:  Z[j1][j2]  = sum_i1 P1[i1][j1] D1[i1][j2]           A = P1^T, prepared; B = D1 as it sits in the
//             accumulators of stage 1 (a lane holds column j2 = lane % 32 and, per 16-row step, the rows
//             8 (e / 4) + 4 (lane / 32) + e % 4), which is a valid B operand once the contraction index of a
//             step is permuted the same way in A.  The tiles of D1 change hands through LDS.
// A tile is 32 x 32 outputs, one wave per tile and stage.
// Precision.  x is fp16 and enters exactly.  An fp32 factor or intermediate v enters as two fp16 numbers,
// hi = fp16(v) and lo = fp16((v - hi) 2^11): v = hi + lo 2^-11 up to 2^-22 |v|, whatever the magnitude of v
// (the factor 2^11 keeps lo out of the subnormal range as long as hi is normal).  Products with hi go to one
// accumulator, the cross products hi lo to a second one that is added with weight 2^-11 at the end; lo lo
// (2^-22) is dropped.  The result is rounded to fp16 once.  Needs |P entries| <= 65504.
// The prepared operands (btc_transform_prepare) are the factors split and laid out once per layer:
//   uint4 P2op[JT][KS2][2][64]   B operand of stage 1: lane (l32, h) of column block c holds P2[16 ks + 8 h + e][32 c + l32]
//   uint4 P1op[IT][KS1][2][64]   A operand of stage 2: lane (l32, h) of row block a holds
//                                P1[16 ks + 8 (e / 4) + 4 h + e % 4][32 a + l32]
// with IT = ceil(n1 / 32), JT = ceil(n2 / 32), KS1 = ceil(n1 / 16), KS2 = n2 / 16 (n2 a multiple of 16), zeros
// outside the matrices, part 0 = hi, part 1 = lo.
#ifndef BTC_FUSED_TRANSFORM_H_
#define BTC_FUSED_TRANSFORM_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace btc {
namespace ftr {

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

struct Geo {
  const uint8_t* sign_bytes;   // bit (i & 7) of byte (i >> 3): sigma[i] = +1 when set
  const uint4* prep;           // P2op, then P1op
  uint16_t* xt_out;            // where workgroup 0 also stores the transformed row (fp16 [n1 n2]), or null
  int n1, n2, IT, JT, KS1, KS2;
};

static inline Geo make_geo(const uint32_t* sign_bits, const void* prep, int n1, int n2) {
  Geo g;
  g.sign_bytes = (const uint8_t*)sign_bits;
  g.prep = (const uint4*)prep;
  g.xt_out = nullptr;
  g.n1 = n1;
  g.n2 = n2;
  g.IT = (n1 + 31) / 32;
  g.JT = (n2 + 31) / 32;
  g.KS1 = (n1 + 15) / 16;
  g.KS2 = n2 / 16;
  return g;
}
static inline size_t prepared_bytes(int n1, int n2) {
  const Geo g = make_geo(nullptr, nullptr, n1, n2);
  return (size_t)(g.JT * g.KS2 + g.IT * g.KS1) * 2 * 64 * 16;
}
// LDS bytes of the exchange area: the tiles of D1 as B operands, [JT][KS1][2][64] uint4
static inline size_t exchange_bytes(int n1, int n2) {
  const Geo g = make_geo(nullptr, nullptr, n1, n2);
  return (size_t)g.JT * g.KS1 * 2 * 64 * 16;
}
constexpr size_t exchange_bytes_c(int n1, int n2) { return (size_t)((n2 + 31) / 32) * ((n1 + 15) / 16) * 2 * 64 * 16; }
// Factor sizes for which a decode kernel with the fused prologue is instantiated (the row must also be the layer's
// input: n1 n2 = in).  The operand layout itself serves any n1 <= 128, n2 <= 128 with n2 a multiple of 16.
static inline bool geometry_ok(int n1, int n2) { return n1 == 64 && (n2 == 64 || n2 == 80); }

__device__ __forceinline__ f32x16 mfma16(const u32x4 a, const u32x4 b, const f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// v -> hi, lo with v = hi + lo 2^-11 (up to 2^-22 |v|)
__device__ __forceinline__ void split2(float v, uint32_t& hi, uint32_t& lo) {
  const _Float16 h = (_Float16)v;
  hi = (uint32_t)__builtin_bit_cast(uint16_t, h);
  lo = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)((v - (float)h) * 2048.0f));
}

// The factor sizes are compile-time constants inside a decode kernel, so that both stages are straight-line code.
// Every workgroup needs ALL operands -- the prepared factors and the row, 56 KB at 64 x 80 -- and each of its tiles
// needs a third of them; fetched per tile that is 138 KB per workgroup through a 64 B/clk L1 and, summed over the
// chip, most of what the L2 can deliver in the time available.  So the workgroup fetches every operand ONCE:
// all NTHR threads copy the prepared buffer and the row into an LDS scratch area (requested when the kernel
// starts -- begin -- and stored when they have arrived), and the tiles read their operands from there.  The row's
// lines are padded by 16 bytes so that the 16-byte reads of 16 consecutive rows hit different banks.
// Waves 0 .. IT JT - 1 take the tiles of stage 1, the next IT JT waves those of stage 2 (one tile each).
template <int N1, int N2, int NTHR>
struct Shared {
  static constexpr int IT = (N1 + 31) / 32, JT = (N2 + 31) / 32, KS1 = (N1 + 15) / 16, KS2 = N2 / 16;
  static constexpr int NT = IT * JT;                    // tiles per stage
  static_assert(N2 % 16 == 0 && N1 >= 1 && N1 <= 128 && N2 <= 128, "factor sizes");
  // the scratch area, in units of 16 bytes: P2op, P1op (as prepared), the row (N2 / 8 + 1 units per line), the
  // tiles of the intermediate
  static constexpr int kPrep = (JT * KS2 + IT * KS1) * 2 * 64;
  static constexpr int kXLine = N2 / 8 + 1;
  static constexpr int kXAt = kPrep, kX = N1 * kXLine;
  static constexpr int kDxAt = kXAt + kX, kDx = JT * KS1 * 2 * 64;
  static constexpr int kScratchBytes = (kDxAt + kDx) * 16;
  static constexpr int kCopy = kPrep + N1 * (N2 / 8);   // units to copy
  static constexpr int LPT = (kCopy + NTHR - 1) / NTHR; // per thread
  struct Ring {
    u32x4 r[LPT];
    uint32_t sg[KS2];
  };

  static __device__ __forceinline__ void begin(const Geo& g, const uint16_t* __restrict__ x, int tid, int wave, int lane,
                                                Ring& R) {
    const u32x4* prep = (const u32x4*)g.prep;
    const u32x4* x4 = (const u32x4*)x;
#pragma unroll
    for (int u = 0; u < LPT; ++u) {
      const int i = tid + u * NTHR;
      const u32x4* src = i < kPrep ? prep + i : x4 + min(i - kPrep, N1 * (N2 / 8) - 1);
      R.r[u] = *src;
    }
    {
      // the signs of this wave's stage-1 tile.  Waves without a tile fetch those of tile 0 and never use them: under
      // a test of the wave number the compiler copies the fetched bytes where the two paths join, i.e. waits for
      // them, and with them for every load requested before them, right here.
      const int a = (wave < NT ? wave : 0) / JT;
      const int i1 = min(a * 32 + (lane & 31), N1 - 1);
#pragma unroll
      for (int u = 0; u < KS2; ++u) R.sg[u] = g.sign_bytes[(i1 * N2 + 16 * u + 8 * (lane >> 5)) >> 3];
    }
  }

  // All waves of the workgroup call this (it holds two workgroup barriers); on return every wave has WRITTEN its
  // part of xf -- the caller's next workgroup barrier makes the row visible.  xf: fp16 [N1 N2] in LDS; S: the
  // scratch area in LDS (kScratchBytes).  R: what begin requested for this thread.
  static __device__ __forceinline__ void transform_row(int tid, int wave, int lane, Ring& R, uint16_t* xf, u32x4* S) {
    const int l32 = lane & 31, h = lane >> 5;
#pragma unroll
    for (int u = 0; u < LPT; ++u) {
      const int i = tid + u * NTHR;
      if (i < kPrep) {
        S[i] = R.r[u];
      } else if (i < kCopy) {
        const int q = i - kPrep, row = q / (N2 / 8), col = q - row * (N2 / 8);
        S[kXAt + row * kXLine + col] = R.r[u];
      }
    }
    __syncthreads();
    if (wave < NT) {                                            // ---- stage 1
      const int a = wave / JT, c = wave - a * JT;
      f32x16 dm, dc;
#pragma unroll
      for (int e = 0; e < 16; ++e) dm[e] = dc[e] = 0.f;
      const int i1 = a * 32 + l32;
      const bool row_ok = i1 < N1;
      const u32x4* ap = S + kXAt + min(i1, N1 - 1) * kXLine + h;
      const u32x4* bp = S + (c * KS2 * 2) * 64 + lane;
#pragma unroll
      for (int u = 0; u < KS2; ++u) {
        const uint32_t minus = ~R.sg[u] & 0xFFu;               // bit e set: element e changes sign
        u32x4 av = ap[2 * u];
        av.x ^= ((minus & 1u) << 15) | ((minus & 2u) << 30);
        av.y ^= ((minus & 4u) << 13) | ((minus & 8u) << 28);
        av.z ^= ((minus & 16u) << 11) | ((minus & 32u) << 26);
        av.w ^= ((minus & 64u) << 9) | ((minus & 128u) << 24);
        if (!row_ok) av = u32x4{0u, 0u, 0u, 0u};
        dm = mfma16(av, bp[u * 128], dm);
        dc = mfma16(av, bp[u * 128 + 64], dc);
      }
      // the tile as B operands of stage 2: step s2 of this row block takes elements 8 s2 .. 8 s2 + 7
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        if (2 * a + s2 < KS1) {
          uint32_t qh[8], ql[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) split2(fmaf(dc[8 * s2 + e], 0x1p-11f, dm[8 * s2 + e]), qh[e], ql[e]);
          u32x4* dst = S + kDxAt + ((c * KS1 + 2 * a + s2) * 2) * 64 + lane;
          dst[0] = u32x4{qh[0] | qh[1] << 16, qh[2] | qh[3] << 16, qh[4] | qh[5] << 16, qh[6] | qh[7] << 16};
          dst[64] = u32x4{ql[0] | ql[1] << 16, ql[2] | ql[3] << 16, ql[4] | ql[5] << 16, ql[6] | ql[7] << 16};
        }
      }
    }
    __syncthreads();
    if (wave >= NT && wave < 2 * NT) {                          // ---- stage 2
      const int a = (wave - NT) / JT, c = (wave - NT) - a * JT;
      const u32x4* ap = S + (JT * KS2 * 2) * 64 + (a * KS1 * 2) * 64 + lane;
      const u32x4* bp = S + kDxAt + (c * KS1 * 2) * 64 + lane;
      f32x16 zm, zc;
#pragma unroll
      for (int e = 0; e < 16; ++e) zm[e] = zc[e] = 0.f;
#pragma unroll
      for (int u = 0; u < KS1; ++u) {
        const u32x4 a0 = ap[u * 128], a1 = ap[u * 128 + 64];
        const u32x4 b0 = bp[u * 128], b1 = bp[u * 128 + 64];
        zm = mfma16(a0, b0, zm);
        zc = mfma16(a1, b0, zc);
        zc = mfma16(a0, b1, zc);
      }
      const int j2 = c * 32 + l32;
      if (j2 < N2) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j1 = a * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
          if (j1 < N1) xf[j1 * N2 + j2] = __builtin_bit_cast(uint16_t, (_Float16)fmaf(zc[e], 0x1p-11f, zm[e]));
        }
      }
    }
  }
};

// not fused: nothing to hold
template <int NTHR>
struct Shared<0, 0, NTHR> {
  struct Ring {};
  static constexpr int NT = 0, kScratchBytes = 0;
};

// Direct: every tile fetches its own operands from global memory into registers -- for the kernel that transforms
// one row by itself (one workgroup per 32 output columns: nothing is shared between its tiles but the row), where
// the scratch area of Shared would not fit (108 x 128).  The factor sizes are compile-time constants, so that both
// stages are straight-line code whose operands are ALL requested when the kernel starts (ring_begin).  The two stages run on different waves: waves 0 .. IT JT - 1 take the tiles of stage 1, the next IT JT waves
// those of stage 2 (one tile each: the workgroup needs 2 IT JT waves).  One register file serves both roles:
// stage 1 holds (a, b hi, b lo) of step u in r[3 u ..], stage 2 (a hi, a lo) in r[2 u ..].
template <int N1, int N2>
struct Direct {
  static constexpr int IT = (N1 + 31) / 32, JT = (N2 + 31) / 32, KS1 = (N1 + 15) / 16, KS2 = N2 / 16;
  static constexpr int NT = IT * JT;                    // tiles per stage
  static constexpr int NR = 3 * KS2 > 2 * KS1 ? 3 * KS2 : 2 * KS1;
  static_assert(N2 % 16 == 0 && N1 >= 1 && N1 <= 128 && N2 <= 128, "factor sizes");
  struct Ring {
    u32x4 r[NR];
    uint32_t sg[KS2];
  };

  static __device__ __forceinline__ void ring_begin(const Geo& g, const uint16_t* __restrict__ x, int wave, int lane, Ring& R) {
    const int l32 = lane & 31, h = lane >> 5;
    if (wave < NT) {
      const int a = wave / JT, c = wave - a * JT;
      const int i1 = min(a * 32 + l32, N1 - 1);                 // rows past the end: a valid row, zeroed when used
      const u32x4* bp = (const u32x4*)g.prep + ((size_t)(c * KS2) * 2) * 64 + lane;
#pragma unroll
      for (int u = 0; u < KS2; ++u) {
        const int k = i1 * N2 + 16 * u + 8 * h;
        R.r[3 * u] = *(const u32x4*)(x + k);
        R.sg[u] = g.sign_bytes[k >> 3];
        R.r[3 * u + 1] = bp[u * 128];
        R.r[3 * u + 2] = bp[u * 128 + 64];
      }
      // (keeps the optimiser from merging the tails of the two branches into stores through a selected address,
      // which would put the ring in scratch memory)
      __builtin_amdgcn_sched_barrier(0);
    } else if (wave < 2 * NT) {
      const int a = (wave - NT) / JT;
      const u32x4* ap = (const u32x4*)g.prep + (size_t)JT * KS2 * 2 * 64 + ((size_t)a * KS1 * 2) * 64 + lane;
#pragma unroll
      for (int u = 0; u < KS1; ++u) {
        R.r[2 * u] = ap[u * 128];
        R.r[2 * u + 1] = ap[u * 128 + 64];
      }
    }
  }

  // All waves of the workgroup call this (it holds one workgroup barrier); on return every wave has WRITTEN its part
  // of xf -- the caller's next workgroup barrier makes the row visible.  xf: fp16 [N1 N2] in LDS; Dx: exchange area
  // in LDS, [JT][KS1][2][64] uint4.  R: what ring_begin requested for this wave.
  static __device__ __forceinline__ void transform_row(int wave, int lane, Ring& R, uint16_t* xf, uint4* Dx) {
    const int l32 = lane & 31, h = lane >> 5;
    if (wave < NT) {                                            // ---- stage 1
      const int a = wave / JT, c = wave - a * JT;
      f32x16 dm, dc;
#pragma unroll
      for (int e = 0; e < 16; ++e) dm[e] = dc[e] = 0.f;
      const bool row_ok = a * 32 + l32 < N1;
#pragma unroll
      for (int u = 0; u < KS2; ++u) {
        const uint32_t minus = ~R.sg[u] & 0xFFu;               // bit e set: element e changes sign
        u32x4 av = R.r[3 * u];
        av.x ^= ((minus & 1u) << 15) | ((minus & 2u) << 30);
        av.y ^= ((minus & 4u) << 13) | ((minus & 8u) << 28);
        av.z ^= ((minus & 16u) << 11) | ((minus & 32u) << 26);
        av.w ^= ((minus & 64u) << 9) | ((minus & 128u) << 24);
        if (!row_ok) av = u32x4{0u, 0u, 0u, 0u};
        dm = mfma16(av, R.r[3 * u + 1], dm);
        dc = mfma16(av, R.r[3 * u + 2], dc);
      }
      // the tile as B operands of stage 2: step s2 of this row block takes elements 8 s2 .. 8 s2 + 7
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        if (2 * a + s2 < KS1) {
          uint32_t qh[8], ql[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) split2(fmaf(dc[8 * s2 + e], 0x1p-11f, dm[8 * s2 + e]), qh[e], ql[e]);
          u32x4* dst = (u32x4*)Dx + ((size_t)(c * KS1 + 2 * a + s2) * 2) * 64 + lane;
          dst[0] = u32x4{qh[0] | qh[1] << 16, qh[2] | qh[3] << 16, qh[4] | qh[5] << 16, qh[6] | qh[7] << 16};
          dst[64] = u32x4{ql[0] | ql[1] << 16, ql[2] | ql[3] << 16, ql[4] | ql[5] << 16, ql[6] | ql[7] << 16};
        }
      }
    }
    __syncthreads();
    if (wave >= NT && wave < 2 * NT) {                          // ---- stage 2
      const int a = (wave - NT) / JT, c = (wave - NT) - a * JT;
      const u32x4* bp = (const u32x4*)Dx + ((size_t)c * KS1 * 2) * 64 + lane;
      f32x16 zm, zc;
#pragma unroll
      for (int e = 0; e < 16; ++e) zm[e] = zc[e] = 0.f;
#pragma unroll
      for (int u = 0; u < KS1; ++u) {
        const u32x4 b0 = bp[u * 128], b1 = bp[u * 128 + 64];
        zm = mfma16(R.r[2 * u], b0, zm);
        zc = mfma16(R.r[2 * u + 1], b0, zc);
        zc = mfma16(R.r[2 * u], b1, zc);
      }
      const int j2 = c * 32 + l32;
      if (j2 < N2) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j1 = a * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
          if (j1 < N1) xf[j1 * N2 + j2] = __builtin_bit_cast(uint16_t, (_Float16)fmaf(zc[e], 0x1p-11f, zm[e]));
        }
      }
    }
  }
};

// not fused: nothing to hold

}  // namespace ftr
}  // namespace btc

#endif  // BTC_FUSED_TRANSFORM_H_
