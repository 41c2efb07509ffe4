// Decode-time product on the 4-bit matrix cores of gfx950.
//
//     y_r = alpha_r * sum_j <x_j, C[I_rj]> + mu_r * sum_k x_k
// (appendix "Binary Codebook LUT-GEMM", blockwise definition of y_r; dequantisation step of
// Algorithm "Binary Transformation and Compression").
//
// A +-1 weight is exactly representable in the 4-bit float format E2M1 (0x2 = +1, 0xA = -1), and an
// fp16 activation is exactly the sum of four E5M2 numbers (E5M2 is the top byte of an fp16: take the top
// byte, subtract, repeat -- every step removes three significant bits and the subtraction is exact).
// So the product of 16 weight rows with one activation row is ONE instruction per 128 weights per row,
//     V_MFMA_F32_16X16X128_F8F6F4   (A = 16 x 128 fp4 weights, B = 128 x 16 bf8, fp32 accumulate),
// with the four pieces of x in four of the sixteen B columns and the result exact up to fp32
// accumulation.  The paper's kernel trades multiplications for table lookups of partial dot products
// because its hardware has no such instruction; here the lookup that remains is the codebook itself:
//
//  * The codebook is expanded once per workgroup into LDS entries of v nibbles (one 8-byte entry per
//    codeword, replicated so that the 16 lanes the LDS serves together read 16 different banks whatever
//    their indices).  A chunk costs one 8-byte LDS read; three chunks (v = 9, 10) are merged by four
//    shift-or operations into the 128-bit A operand of a lane.  No per-column table is ever built.
//  * The contraction index of an MFMA may be permuted freely as long as both operands agree.  Lane
//    (row r, k block q) of wave w owns a contiguous run of G*T chunks of row r ("strand" 4w + q), G =
//    floor(32 / v) chunks per operand and T instructions per row block, so its index bits are one
//    contiguous piece of the row's stream: a few 16-byte loads, one funnel shift to normalise, and every
//    field sits at a compile-time position.  The B operands follow the same permutation; they depend on x
//    only, are built once per workgroup (through an LDS staging area, in operand layout) and then live
//    in registers for all row blocks the workgroup walks.  One activation row fills 4 of the 16 B
//    columns, so one set of B registers serves FOUR steps: columns 4c..4c+3 hold the pieces of step
//    4 tt + c, step 4 tt + c accumulates into accumulator c, and only columns 4c..4c+3 of accumulator c
//    are kept at the end (the other columns are products with another step's activations).
//  * A workgroup owns whole rows: its W waves split the columns, their sixteen-row partial sums meet in
//    LDS (one barrier per row block, double-buffered) and one wave applies alpha, mu * sum(x) and stores.
//    No workspace, no traffic between workgroups, one launch, deterministic.
//  * Index words are requested three row blocks ahead; a row block is 16 whole rows of the stream, so
//    the matrix is read front to back in large contiguous pieces.
#include <hip/hip_fp16.h>

#include <cstdlib>
#include <type_traits>

#include "btc_internal.h"

namespace btc {
namespace fp4 {

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((address_space(3))) unsigned long long lds_u64;

constexpr uint32_t kOob = 0x80000000u;   // buffer offset that is always out of range (buffers are < 2 GiB)
constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format
constexpr int kPD = 4;                   // row blocks in flight per wave (the row loop is unrolled by this)
constexpr int kSetBytes = 512;           // staged B operand of one step: 4 pieces x 4 k blocks x 32 bytes

template <int V, int B, int T, int W>
struct Cfg {
  static constexpr int G = 32 / V;                          // chunks per 128-bit operand of a lane
  static constexpr int EW = 4 * V;                          // bits of a table entry
  static constexpr int L = G * T;                           // chunks per strand
  static constexpr int ND = (L * B + 31) / 32 + 1;          // index words a lane needs per row block
  // index words of a wave's four strands inside one row, fetched as 16-byte pieces by LPR lanes per row
  static constexpr int NW = (4 * L * B + 31) / 32 + 1;
  static constexpr int LPR = (NW + 3) / 4;
  static constexpr int RPI = 64 / LPR;                      // rows per load instruction
  static constexpr int NLD = (16 + RPI - 1) / RPI;          // load instructions per row block
  static constexpr int S = 4 * LPR + 4;                     // staged row stride in words
  static constexpr int C = (B == 8) ? 32 : (B <= 9) ? 16 : (B == 10 ? 8 : (B == 11 ? 4 : (B == 12 ? 2 : 1)));  // table copies
  static constexpr int LOG2C = C == 32 ? 5 : C == 16 ? 4 : (C == 8 ? 3 : (C == 4 ? 2 : (C == 2 ? 1 : 0)));
  static constexpr int kTableBytes = (1 << B) * C * 8;
  static constexpr int kRedBytes = (4 * W * 16 * 4 + W * 4 + 15) & ~15;
  static constexpr int kIdxBytes = W * 2 * 16 * S * 4;      // two staged row blocks per wave
  static constexpr int kStageBytes = W * T * kSetBytes;
  static constexpr int kLdsBytes = kTableBytes + kRedBytes + kIdxBytes + kStageBytes;
  static constexpr int kWavesPerEu = (T <= 5 && kLdsBytes <= 80 * 1024 - 64) ? 2 * W / 4 : W / 4;
  static_assert(V >= 5 && V <= 16, "one 8-byte entry per codeword");
  static_assert(LPR <= 32, "at least two rows per load instruction");
};

__device__ __forceinline__ float dpp_xor1(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_xor2(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
}
// Sum over the 64 lanes, valid in lane 63.
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  v += dpp_xor1(v);
  v += dpp_xor2(v);
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false)); // row_bcast:15
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false)); // row_bcast:31
  return v;
}

// LDS operations of one wave complete in issue order; keep the compiler from moving accesses across this
// point, so that lanes may read what other lanes of the same wave wrote before it.
__device__ __forceinline__ void wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Codeword (bit t = element t, 1 => +1) -> V nibbles, 0x2 = +1.0 and 0xA = -1.0 in E2M1.
template <int V>
__device__ __forceinline__ unsigned long long expand_codeword(uint32_t c) {
  unsigned long long e = 0;
#pragma unroll
  for (int t = 0; t < V; ++t) e |= (unsigned long long)(((c >> t) & 1u) ? 0x2u : 0xAu) << (4 * t);
  return e;
}

#ifdef BTC_FP4_STAMPS
__device__ unsigned long long g_stamps[4 * 64];
#define STAMP(i)                                                                                   \
  do {                                                                                             \
    if (tid == 0 && (blockIdx.x == 0 || blockIdx.x == gridDim.x / 2 || blockIdx.x == gridDim.x - 1)) \
      g_stamps[(blockIdx.x == 0 ? 0 : (blockIdx.x == gridDim.x - 1 ? 2 : 1)) * 64 + (i)] = wall_clock64(); \
  } while (0)
#else
#define STAMP(i)
#endif

template <int V, int B, int T, int W>
__global__ __launch_bounds__(W * 64, (Cfg<V, B, T, W>::kWavesPerEu)) void gemv_fp4_kernel(
    Dims d, const uint32_t* __restrict__ packed, const uint32_t* __restrict__ codebook,
    const float* __restrict__ alpha, const float* __restrict__ mu, const __half* __restrict__ x,
    void* __restrict__ y, int y_is_f32, int n_rb, int x_dword) {
  using K = Cfg<V, B, T, W>;
  constexpr int G = K::G, EW = K::EW, ND = K::ND, C = K::C, L = K::L;
  constexpr int LPR = K::LPR, RPI = K::RPI, NLD = K::NLD, S = K::S;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned long long* table = (unsigned long long*)smem;                       // [2^B][C], at LDS offset 0
  float* red = (float*)(smem + K::kTableBytes);                                // [2 phases][2 row blocks][W][16]
  float* sxp = red + 4 * W * 16;                                               // [W]
  uint32_t* idx_all = (uint32_t*)(smem + K::kTableBytes + K::kRedBytes);       // [W][2 row blocks][16][S]
  unsigned char* bstage_all = smem + K::kTableBytes + K::kRedBytes + K::kIdxBytes;  // [W][T][512]

  const int tid = threadIdx.x, lane = tid & 63;
  STAMP(0);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, q = lane >> 4;
  const int stride = gridDim.x;

  // ---- small loads first (their data is needed first): codewords, this wave's activations.
  // An item is 16 consecutive B bytes of one step: (step t, strand qa, half h) = slots e = 16 h .. 16 h + 15
  // of strand qa, which are the CONSECUTIVE elements (chunk0(qa) + G t) * V + e of x for e < G * V (the
  // G chunks of a step follow one another in x) and padding above.  Slot k = 32 qa + e of an instruction
  // sits in B lane k block q' = 2 (qa & 1) + (e >> 4) at byte 16 (qa >> 1) + (e & 15).
  constexpr int KPT = ((1 << B) + W * 64 - 1) / (W * 64);
  uint32_t cw[KPT];
#pragma unroll
  for (int i = 0; i < KPT; ++i) cw[i] = codebook[min(tid + i * W * 64, (1 << B) - 1)];
  unsigned char* bstage = bstage_all + wave * (T * kSetBytes);
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, d.in * 2, kRsrcFlags);
  constexpr int n_items = 8 * T;
  constexpr int NI = (n_items + 63) / 64;
  uint32_t hx[NI][8];                                      // 16 fp16 values per item
#pragma unroll
  for (int ii = 0; ii < NI; ++ii) {
    const int item = lane + 64 * ii;
    const int t = item >> 3, qa = (item >> 1) & 3, h = item & 1;
    const uint32_t x0 = (uint32_t)((wave * 4 + qa) * L + G * t) * V + 16u * h;   // first element of the item
    const bool live = item < n_items;
    if (x_dword) {        // x0 is even: two 16-byte loads (4-byte aligned), range-checked word by word
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const auto v4 = __builtin_amdgcn_raw_buffer_load_b128(rx, live ? (x0 + 8u * i) * 2u : kOob, 0, 0);
#pragma unroll
        for (int k = 0; k < 4; ++k) hx[ii][4 * i + k] = (16 * h + 8 * i + 2 * k < G * V) ? v4[k] : 0u;   // padding slots
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t lo = __builtin_amdgcn_raw_buffer_load_b16(rx, (live && 16 * h + 2 * i < G * V) ? (x0 + 2u * i) * 2u : kOob, 0, 0);
        const uint32_t hi = __builtin_amdgcn_raw_buffer_load_b16(rx, (live && 16 * h + 2 * i + 1 < G * V) ? (x0 + 2u * i + 1) * 2u : kOob, 0, 0);
        hx[ii][i] = (lo & 0xFFFFu) | (hi << 16);
      }
    }
  }

  // ---- index words.  The wave's four strands are one contiguous piece of every row: LPR lanes fetch it as
  // 16-byte pieces (neighbouring lanes read neighbouring addresses), RPI rows per instruction; the pieces go
  // through a wave-private LDS area from which lane (row r, strand q) reads its own run of words.
  const uint32_t wbit0 = (uint32_t)(wave * 4 * L) * B;       // first bit of the wave's piece inside a row
  const int wd0 = (int)(wbit0 >> 5);
  const int lrow = lane / LPR, lpc = lane - lrow * LPR;
  const uint32_t row_bytes = (uint32_t)d.wpr * 4u;
  const uint32_t total_bytes = (uint32_t)d.out * row_bytes;
  const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc((void*)packed, 0, (int)total_bytes, kRsrcFlags);
  // the whole byte offset is per-lane: that is the part the hardware checks against the buffer size, word
  // by word (a piece that runs past the end of the last row reads zeros)
  const uint32_t piece_off = (lrow < RPI && wd0 + 4 * lpc < d.wpr) ? (uint32_t)(wd0 + 4 * lpc) * 4u : kOob;
  uint4 D[kPD][NLD];
  auto load_block = [&](int rb, uint4 (&dst)[NLD]) {
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      const int rr = j * RPI + lrow;
      const int row = rb * 16 + rr;
      const uint32_t off = (rb < n_rb && rr < 16 && row < d.out && piece_off != kOob) ? (uint32_t)row * row_bytes + piece_off : kOob;
      const auto v4 = __builtin_amdgcn_raw_buffer_load_b128(rp, off, 0, 0);
      dst[j] = make_uint4(v4[0], v4[1], v4[2], v4[3]);
    }
  };
  uint32_t* idx_stage = idx_all + wave * (2 * 16 * S);
  auto stage_block = [&](int parity, const uint4 (&src)[NLD]) {
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      const int rr = j * RPI + lrow;
      if (lrow < RPI && rr < 16) *(uint4*)(idx_stage + (parity * 16 + rr) * S + 4 * lpc) = src[j];
    }
  };
#pragma unroll
  for (int u = 0; u < kPD; ++u) load_block(blockIdx.x + u * stride, D[u]);
  STAMP(1);

  // ---- codebook -> table of nibble patterns, every entry C times.  Thread k writes its entry's copies in
  // the order k, k + 1, ... (mod C): at every step the 16 threads of consecutive entries write 16 different
  // bank pairs, although an entry's copies are 128 bytes apart from the next entry's.
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    const int k = tid + i * W * 64;
    if (k < (1 << B)) {
      const unsigned long long ent = expand_codeword<V>(cw[i]);
#pragma unroll
      for (int c = 0; c < C; ++c) table[k * C + ((c + k) & (C - 1))] = ent;
    }
  }
  STAMP(2);

  // ---- activations -> four E5M2 pieces each (the top byte of an fp16 IS an E5M2 number; subtracting it
  // leaves at most 8 significant bits, exactly), written in B-operand layout: 16 bytes per item and piece
  float sx_lane = 0.f;
#pragma unroll
  for (int ii = 0; ii < NI; ++ii) {
    const int item = lane + 64 * ii;
    const int t = item >> 3, qa = (item >> 1) & 3, h = item & 1;
    unsigned char* dst = bstage + t * kSetBytes + (2 * (qa & 1) + h) * 32 + 16 * (qa >> 1);
    uint32_t res[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      res[i] = hx[ii][i];
      const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
      sx_lane = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, res[i]), one, sx_lane, false);
    }
    if (item < n_items) {
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        uint32_t o4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)   // bytes 1 and 3 of two dwords: the pieces of four consecutive elements
          o4[j] = __builtin_amdgcn_perm(res[2 * j + 1], res[2 * j], 0x07050301u);
        *(uint4*)(dst + n * 128) = make_uint4(o4[0], o4[1], o4[2], o4[3]);
        if (n < 3) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const f16x2 top = __builtin_bit_cast(f16x2, res[i] & 0xFF00FF00u);
            res[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, res[i]) - top);
          }
        }
      }
    }
  }
  STAMP(5);
  // sum of this wave's activations (every element belongs to exactly one item)
  sx_lane = wave_sum_to_lane63(sx_lane);
  if (lane == 63) sxp[wave] = sx_lane;
  wave_lds_order();

  // ---- B operands of this wave: lane (column n, k block q) of set t holds piece n of step t for n < 4
  // and zeros in the other columns
  i32x8 Bq[T];
#pragma unroll
  for (int t = 0; t < T; ++t) {
    Bq[t] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
    if (r < 4) {
      const uint4* src = (const uint4*)(bstage + t * kSetBytes + r * 128 + q * 32);
      const uint4 lo = src[0], hi = src[1];
      Bq[t] = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    }
  }
  // the first pair of row blocks: index words -> LDS, registers refilled with the third pair's
  stage_block(0, D[0]);
  stage_block(1, D[1]);
  load_block(blockIdx.x + 4 * stride, D[0]);
  load_block(blockIdx.x + 5 * stride, D[1]);
  STAMP(6);
  __syncthreads();   // table complete, sums of x stored
  STAMP(7);
  float sx = 0.f;
#pragma unroll
  for (int w = 0; w < W; ++w) sx += sxp[w];

  // ---- per-lane constants of the read-back: lane (r, q) starts at bit ws0 + q L B of its staged row
  const uint32_t lbit = (wbit0 & 31u) + (uint32_t)(q * L) * B;
  const uint32_t s0 = lbit & 31u;
  const uint32_t* my_words = idx_stage + r * S + (lbit >> 5);
  const uint32_t lane_copy = (uint32_t)(lane & (C - 1)) * 8u;   // this lane's copy of every table entry
  // ---- the row loop: two row blocks at a time (their instruction streams interleave, so one hides the
  // other's LDS latency; the B registers serve both), one barrier per pair
  int it = 0;
  for (int rb0 = blockIdx.x; rb0 < n_rb; rb0 += 4 * stride) {
#pragma unroll
    for (int pp = 0; pp < 2; ++pp) {
      const int rbA = rb0 + 2 * pp * stride, rbB = rbA + stride;     // rbB may be past the end: zeros, not stored
      if (rbA >= n_rb) break;
      // the waves that will finish the two row blocks ask for their scales now
      const int fwA = it % W, fwB = (it + 1) % W;
      const int my_rb = wave == fwA ? rbA : rbB;
      const int my_row = my_rb * 16 + lane;
      const bool finishes = (wave == fwA || wave == fwB) && lane < 16 && my_rb < n_rb && my_row < d.out;
      float al = 0.f, mm = 0.f;
      if (finishes) {
        al = alpha[my_row];
        mm = mu[my_row];
      }
      // both row blocks' words from LDS; then the next pair's words take their place (LDS operations of a
      // wave complete in order) and the registers are refilled with the pair after that
      wave_lds_order();
      uint32_t Wd[2][ND + 1];
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i <= ND; ++i) Wd[h][i] = my_words[h * 16 * S + i];
      if (it < 4) STAMP(40 + 3 * it);
      wave_lds_order();
      stage_block(0, D[2 * (pp ^ 1)]);
      stage_block(1, D[2 * (pp ^ 1) + 1]);
      if (it < 4) STAMP(41 + 3 * it);
      load_block(rbA + 6 * stride, D[2 * (pp ^ 1)]);
      load_block(rbA + 7 * stride, D[2 * (pp ^ 1) + 1]);
      if (it < 16) STAMP(13 + 3 * it);
      uint32_t R[2][ND];     // normalised: bit 0 is the first bit of the lane's run
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < ND; ++i) R[h][i] = __builtin_amdgcn_alignbit(Wd[h][i + 1], Wd[h][i], s0);
      if (it < 16) STAMP(8 + 3 * it);

      // The step loop, software-pipelined by hand: the table reads of step t + 1 (both row blocks) are issued
      // before the entries of step t are merged and contracted, so an LDS round trip is covered by a step's
      // worth of arithmetic.  (Left to itself the compiler waits for every group of three reads.)
      f32x4 acc[2][2] = {{{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}};
      unsigned long long E[2][2][G];   // [pipeline stage][row block][chunk]
      auto issue = [&](int t, unsigned long long (&dst)[2][G]) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const int pos = (t * G + g) * B, w = pos >> 5, sb = pos & 31;
            uint32_t ofs;
            if (B == 8 && C == 32) {
              // byte-aligned indices, one table copy per lane pair of banks: offset = index << 8 | copy,
              // assembled by one byte permute
              ofs = __builtin_amdgcn_perm(R[h][w], lane_copy, 0x0C0C0000u | ((4u + (sb >> 3)) << 8));
            } else {
              // table offset of the entry = index << SH | copy: the field is extracted already shifted
              constexpr int SH = 3 + K::LOG2C;
              constexpr uint32_t mask = ((1u << B) - 1u) << SH;
              uint32_t sh;
              if (sb + B <= 32) sh = sb >= SH ? R[h][w] >> (sb - SH) : R[h][w] << (SH - sb);
              else sh = sb >= SH ? __builtin_amdgcn_alignbit(R[h][w + 1], R[h][w], sb - SH)
                                 : __builtin_amdgcn_alignbit(R[h][w + 1], R[h][w], sb) << SH;
              ofs = (sh & mask) | lane_copy;
            }
            // the table starts at LDS address 0 (this kernel has no static LDS), so the offset IS the address
            dst[h][g] = *(const lds_u64*)(uintptr_t)ofs;
          }
      };
      auto consume = [&](int t, const unsigned long long (&src)[2][G]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          uint32_t A[4] = {0u, 0u, 0u, 0u};
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const uint32_t lo = (uint32_t)src[h][g], hi = (uint32_t)(src[h][g] >> 32);
            const int bit = g * EW, w0 = bit >> 5, ss = bit & 31;
            if (ss == 0) {
              A[w0] |= lo;
              if (EW > 32) A[w0 + 1] |= hi;
            } else {
              A[w0] |= lo << ss;
              if (EW + ss > 32) A[w0 + 1] |= __builtin_amdgcn_alignbit(hi, lo, 32 - ss);
              if (EW + ss > 64) A[w0 + 2] |= hi >> (32 - ss);
            }
          }
          const i32x8 Av = {(int)A[0], (int)A[1], (int)A[2], (int)A[3], 0, 0, 0, 0};
          acc[h][t & 1] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(Av, Bq[t], acc[h][t & 1], 4 /* A: E2M1 */,
                                                                           1 /* B: E5M2 */, 0, 0, 0, 0);
        }
      };
      issue(0, E[0]);
#pragma unroll
      for (int t = 0; t < T; ++t) {
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < T) issue(t + 1, E[(t + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        consume(t, E[t & 1]);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (it < 16) STAMP(9 + 3 * it);
      // columns 0..3 hold the four pieces' sums, the other columns are zero: add the quad, lane 0 of a row
      // group stores its four rows
      float* rbuf = red + pp * (2 * W * 16);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        float s4[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v = acc[h][0][i] + acc[h][1][i];
          v += dpp_xor1(v);
          v += dpp_xor2(v);
          s4[i] = v;
        }
        if (r == 0) *(float4*)(rbuf + h * (W * 16) + wave * 16 + 4 * q) = make_float4(s4[0], s4[1], s4[2], s4[3]);
      }
      if (it < 16) STAMP(10 + 3 * it);
      __syncthreads();
      if (it < 16) STAMP(11 + 3 * it);
      if (finishes) {
        const float* fb = rbuf + (wave == fwA ? 0 : W * 16);
        float tot = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) tot += fb[w * 16 + lane];
        const float res = al * tot + mm * sx;
        if (y_is_f32) ((float*)y)[my_row] = res;
        else ((__half*)y)[my_row] = __float2half_rn(res);
      }
      if (it < 16) STAMP(12 + 3 * it);
      it += 2;
    }
  }
  STAMP(63);
}

constexpr int kLdsMax = 160 * 1024 - 64;

template <int V, int B, int T, int W>
static btc_status launch3(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                          const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  using K = Cfg<V, B, T, W>;
  if constexpr (K::kLdsBytes > kLdsMax) {
    return BTC_ERR_UNSUPPORTED;
  } else {
    static bool attr_set = false;   // one-time kernel attribute, not call state
    if (!attr_set) {
      if (hipFuncSetAttribute((const void*)gemv_fp4_kernel<V, B, T, W>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              K::kLdsBytes) != hipSuccess)
        return BTC_ERR_HIP;
      attr_set = true;
    }
    const int n_rb = (d.out + 15) / 16;
    const int per_cu = K::kWavesPerEu * 4 / W;           // workgroups resident per compute unit (registers, LDS)
    const int slots = 256 * per_cu;
    const int grid = n_rb < slots ? n_rb : slots;        // workgroup i walks row blocks i, i + grid, ...
    const int x_dword = (V % 2 == 0) && (d.in % 2 == 0);
    gemv_fp4_kernel<V, B, T, W><<<grid, W * 64, K::kLdsBytes, q>>>(d, packed, codebook, alpha, mu, (const __half*)x,
                                                                          y, y_is_f32, n_rb, x_dword);
    return launch_status();
  }
}

// Steps per row block: the 4 W strands of a workgroup must cover the row.  Instantiated for a few step counts; a
// strand that is longer than needed reads zeros for the activations past the end of the row.
constexpr int kW = 8;
static int steps_for(const Dims& d) {
  const int G = 32 / d.v;
  const int need = (d.nchunks + kW * 4 * G - 1) / (kW * 4 * G);
  static const int have[] = {3, 4, 5, 6, 8, 9, 10, 12, 15, 16};
  for (int t : have) if (need <= t) return t;
  return 0;
}

template <int V, int B>
static btc_status launch2(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                          const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
#define BTC_FP4_CASE(TT) \
  case TT: return launch3<V, B, TT, kW>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
  switch (steps_for(d)) {
    BTC_FP4_CASE(3) BTC_FP4_CASE(4) BTC_FP4_CASE(5) BTC_FP4_CASE(6) BTC_FP4_CASE(8) BTC_FP4_CASE(9)
    BTC_FP4_CASE(10) BTC_FP4_CASE(12) BTC_FP4_CASE(15) BTC_FP4_CASE(16)
  }
#undef BTC_FP4_CASE
  return BTC_ERR_UNSUPPORTED;
}

template <int V>
static btc_status launch1(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                          const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  switch (d.b) {
    case 7: return launch2<V, 7>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 8: return launch2<V, 8>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 9: return launch2<V, 9>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 10: return launch2<V, 10>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
  }
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace fp4

#ifdef BTC_FP4_STAMPS
extern "C" int btc_debug_fp4_stamps(unsigned long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(fp4::g_stamps), sizeof(unsigned long long) * n);
}
#endif

bool gemv_fp4_covers(const Dims& d) {
  if (d.v != 9 && d.v != 10) return false;
  if (d.b < 7 || d.b > 10) return false;
  if ((long long)d.out * d.wpr * 4 >= (1LL << 31)) return false;
  if ((long long)d.nchunks * d.v * 2 >= (1LL << 31)) return false;
  return fp4::steps_for(d) != 0;    // table (at most 64 KB) + staging (at most 64 KB) always fit
}

btc_status gemv_fp4(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  if (!gemv_fp4_covers(d)) return BTC_ERR_UNSUPPORTED;
  if (d.v == 9) return fp4::launch1<9>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
  return fp4::launch1<10>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
}

}  // namespace btc
