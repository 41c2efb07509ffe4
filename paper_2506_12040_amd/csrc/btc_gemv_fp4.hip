// Decode-time product on the 4-bit matrix cores of gfx950.
//
//     y_r = alpha_r * sum_j <x_j, C[I_rj]> + mu_r * sum_k x_k
// (appendix "Binary Codebook LUT-GEMM", blockwise definition of y_r; dequantisation step of
// Algorithm "Binary Transformation and Compression").
//
// A +-1 weight is exactly representable in the 4-bit float format E2M1 (0x2 = +1, 0xA = -1), and an
// fp16 activation is the sum of four E5M2 numbers (E5M2 is the top byte of an fp16: take the top byte,
// subtract, repeat -- every step removes three significant bits and the subtraction is exact; what could
// be lost is only what falls below the smallest E5M2 number, 2^-16, so every block of activations is first
// multiplied by a power of two that brings its largest element to 2^14..2^15, and the partial sums of that
// block are multiplied by the inverse power afterwards: exact down to 2^-30 of the block's largest
// element).
// So the product of 16 weight rows with one activation row is ONE instruction per 128 weights per row,
//     V_MFMA_F32_16X16X128_F8F6F4   (A = 16 x 128 fp4 weights, B = 128 x 16 bf8, fp32 accumulate),
// with the four pieces of x in four of the sixteen B columns and the result exact up to fp32
// accumulation.  The paper's kernel trades multiplications for table lookups of partial dot products
// because its hardware has no such instruction; here the lookup that remains is the codebook itself:
//
//  * The codebook is expanded once per workgroup into LDS entries of nibbles (one 8-byte entry per
//    codeword: elements 0..7 in the low word, the remaining v - 8 in the high word; every entry is
//    replicated so that the 16 lanes the LDS serves together read 16 different bank pairs whatever their
//    indices).  A chunk costs one 8-byte LDS read.  The contraction index of an MFMA may be permuted freely
//    as long as both operands agree, so a lane's 128-bit A operand is laid out for cheapness: words 0..2
//    ARE the low words of its three chunks, word 3 collects the three short tails (two shift-or operations).
//    No per-column table is ever built.
//  * Lane (row r, k block q) of column wave cw owns a contiguous run of G*T chunks of row r ("strand"
//    4 cw + q), G = floor(32 / v) chunks per operand and T instructions per row block, so its index bits
//    are one contiguous piece of the row's stream and every field sits at a compile-time position after one
//    funnel shift.  The pieces of the 16 rows are fetched by neighbouring lanes from neighbouring
//    addresses (16 bytes each) and handed to their owners through a wave-private LDS area.
//  * The B operands follow the same permutation; they depend on x only, are built once per workgroup (in
//    LDS, in operand layout) and then live in registers.  One activation row fills 4 of the 16 B columns,
//    so one set of eight B registers serves FOUR steps: columns 4c..4c+3 hold the pieces of step 4 tt + c,
//    that step accumulates into accumulator c, and only columns 4c..4c+3 of accumulator c are kept at the
//    end (the other columns are products with another step's activations).  That keeps the kernel below
//    128 registers: four waves per SIMD, which is what hides the LDS and memory latencies here.
//  * A workgroup owns whole rows: eight column waves split the columns of a row block, their sixteen-row
//    partial sums meet in LDS and one wave applies alpha, mu * sum(x) and stores.  Two such teams of eight
//    waves work on two row blocks at a time and share the table, the B operands and one barrier per step
//    of the row loop.  No workspace, no traffic between workgroups, one launch, deterministic.
//  * Index words are requested two row blocks ahead; a row block is 16 whole rows of the stream, so
//    the matrix is read front to back in large contiguous pieces.
#include <hip/hip_fp16.h>

#include <cstdlib>
#include <type_traits>

#include "btc_fused_transform.h"
#include "btc_internal.h"

namespace btc {
namespace fp4 {

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((address_space(3))) u32x2 lds_u32x2;

constexpr uint32_t kOob = 0x80000000u;   // buffer offset that is always out of range (buffers are < 2 GiB)
constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format
constexpr int kSetBytes = 2048;          // B operands of four steps: 16 columns x 4 k blocks x 32 bytes

// CW column waves per team: 8, two teams (LDS permitting) -- or 16 in one team for rows of more than 15360
// weights ("wide"), where every wave prepares its own B operands, one set at a time, in a small buffer.
constexpr int kLdsMax = 160 * 1024 - 64;

// FUSED: the kernel first computes the transformed activation row into an LDS area of its own (fp16, the whole
// reach of the strands, zeros past the end of the row) and takes its activations from there; the table then gets
// as many copies as still fit.
template <int V, int B, int T, int TEAMS, int CW, int GN1 = 0, int GN2 = 0>
struct Cfg {
  static constexpr bool FUSED = GN1 > 0;
  static constexpr int W = CW * TEAMS;                      // waves per workgroup
  static constexpr bool WIDE = CW == 16;
  static constexpr int G = 3;                               // chunks per 128-bit operand of a lane
  static constexpr int TAIL = V - 8;                        // elements of a chunk in the high word of its entry
  static constexpr int L = G * T;                           // chunks per strand
  // Row blocks in flight per wave in registers (one more sits in LDS).  One: measured against two and three, fewer
  // requests in flight are FASTER here (28672 x 8192: 13.9 / 14.3 / 15.2 us with 1 / 2 / 3) -- a wave's later row
  // blocks otherwise queue in front of the blocks other waves need first.
  static constexpr int PD = 1;
  static constexpr int ND = (L * B + 31) / 32 + 1;          // index words a lane needs per row block
  // index words of a wave's four strands inside one row, fetched as 16-byte pieces by LPR lanes per row
  static constexpr int NW = (4 * L * B + 31) / 32 + 1;
  static constexpr int LPR = (NW + 3) / 4;
  static constexpr int RPI = 64 / LPR;                      // rows per load instruction
  static constexpr int NLD = (16 + RPI - 1) / RPI;          // load instructions per row block
  static constexpr int S = 4 * ((LPR + 1) | 1);             // staged row stride in words: an odd number of 16-byte
                                                            // pieces, so that the 16 rows start in 16 different banks
  static constexpr int kRedBytes = (2 * W * 16 * 4 + W * 4 + CW * 2 * 4 + 15) & ~15;
  static constexpr int kIdxBytes = W * 16 * S * 4;          // one staged row block per wave
  static constexpr int NSET = (T + 3) / 4;                  // B register sets
  static constexpr int kStageBytes = WIDE ? 0 : CW * NSET * kSetBytes;   // wide: the wave's index area serves first
  static_assert(!WIDE || 16 * S * 4 >= kSetBytes, "a set fits the wave's index area");
  static constexpr int kXfElems = CW * 4 * L * V;           // elements the strands of a team reach
  static constexpr int kXfBytes = FUSED ? ((kXfElems * 2 + 15) & ~15) : 0;
  // the index and staging areas; FUSED: before they are used, the scratch area of the transform (all its operands
  // and the tiles of its intermediate), which may be larger
  static constexpr int kTrBytes = ftr::Shared<GN1, GN2, CW * TEAMS * 64>::kScratchBytes;
  static constexpr int kWorkBytes = kIdxBytes + kStageBytes > kTrBytes ? kIdxBytes + kStageBytes : kTrBytes;
  static constexpr int kRestBytes = kRedBytes + kWorkBytes + kXfBytes;
  static constexpr int C0 = (B <= 8) ? 32 : (B == 9) ? 16 : 8;  // table copies (32: no two lanes of a wave share a bank pair)
  static constexpr bool fits(int c) { return (1 << B) * c * 8 + kRestBytes <= kLdsMax; }
  static constexpr int C = (!FUSED || fits(C0)) ? C0 : (C0 >= 16 && fits(C0 / 2)) ? C0 / 2 : (C0 >= 32 && fits(C0 / 4)) ? C0 / 4 : C0;
  static constexpr int LOG2C = C == 32 ? 5 : (C == 16 ? 4 : 3);
  static constexpr int kTableBytes = (1 << B) * C * 8;
  static constexpr int kLdsBytes = kTableBytes + kRestBytes;
  static_assert(V == 9 || V == 10, "three chunks per operand, tails of one or two elements");
  static_assert(B >= 7 && B <= 10, "table of at most 64 KB");
  static_assert(LPR <= 32, "at least two rows per load instruction");
  static_assert(TEAMS == 1 || CW == 8, "two teams of eight");
};

__device__ __forceinline__ float dpp_xor1(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_xor2(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_ror4(float v) {   // rotate right by 4 inside a row of 16 lanes
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_ror8(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xF, 0xF, true));
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

// Maximum over the 64 lanes, valid in lane 63.
__device__ __forceinline__ uint32_t wave_max_to_lane63(uint32_t v) {
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true));    // quad xor 1
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true));    // quad xor 2
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true));   // row_half_mirror
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true));   // row_mirror
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false));  // row_bcast:15
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false));  // row_bcast:31
  return v;
}

// LDS operations of one wave complete in issue order; keep the compiler from moving accesses across this
// point, so that lanes may read what other lanes of the same wave wrote before it.
__device__ __forceinline__ void wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Codeword (bit t = element t, 1 => +1) -> nibbles 0x2 = +1.0, 0xA = -1.0 (E2M1): elements 0..7 in the low
// word, elements 8..V-1 in the low bits of the high word.
template <int V>
__device__ __forceinline__ unsigned long long expand_codeword(uint32_t c) {
  uint32_t lo = 0, hi = 0;
#pragma unroll
  for (int t = 0; t < 8; ++t) lo |= (((c >> t) & 1u) ? 0x2u : 0xAu) << (4 * t);
#pragma unroll
  for (int t = 8; t < V; ++t) hi |= (((c >> t) & 1u) ? 0x2u : 0xAu) << (4 * (t - 8));
  return ((unsigned long long)hi << 32) | lo;
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

// Slot e (0..31) of a lane's operand at step t holds element (chunk c, position u) of its three chunks:
// e < 24: c = e / 8, u = e % 8;  24 <= e < 24 + 3 TAIL: c = (e - 24) / TAIL, u = 8 + (e - 24) % TAIL;  else padding.
// The same order is used for the activations on the B side.

// The matrices of one launch: up to kMaxMulti matrices with rows of the same length (same chunk length and codebook
// size; the number of rows may differ) applied to the same activation row -- the q, k, v or the gate, up projections
// of a decoder layer.  Workgroups first[m] .. first[m + 1] - 1 work on matrix m (first[m] = the grid size for the
// slots past `count`); out[m] = its rows (0 on the host side: the rows of the shape handed to the launch).
constexpr int kMaxMulti = 4;
struct Multi {
  const uint32_t* packed[kMaxMulti];
  const uint32_t* codebook[kMaxMulti];
  const float* alpha[kMaxMulti];
  const float* mu[kMaxMulti];
  void* y[kMaxMulti];
  int out[kMaxMulti];
  int first[kMaxMulti + 1];
  int count;
};
struct Extra {
  ftr::Geo geo;
  Multi multi;
};

// GN1, GN2: factor sizes of the activation transform computed in front of the product (0, 0: none).
template <int V, int B, int T, int TEAMS, int CW, int GN1, int GN2>
__global__ __launch_bounds__(CW * TEAMS * 64) void gemv_fp4_kernel(
    Dims d_arg, Multi mm, const __half* __restrict__ x_arg, int y_is_f32, int x_dword_arg, ftr::Geo geo) {
  constexpr bool FUSED = GN1 > 0;
  using K = Cfg<V, B, T, TEAMS, CW, GN1, GN2>;
  using FT = ftr::Shared<GN1, GN2, CW * TEAMS * 64>;
  constexpr int FT_NT = FT::NT;                               // tiles per stage of the transform
  static_assert(!FUSED || V == 10, "the fused prologue reads aligned pairs of activations from LDS");
  constexpr bool WIDE = K::WIDE;
  constexpr int W = K::W, G = K::G, TAIL = K::TAIL, ND = K::ND, C = K::C, L = K::L;
  constexpr int LPR = K::LPR, RPI = K::RPI, NLD = K::NLD, S = K::S, kPD = K::PD;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned long long* table = (unsigned long long*)smem;                       // [2^B][C], at LDS offset 0
  float* red = (float*)(smem + K::kTableBytes);                                // [2 phases][W][16]
  float* sxp = red + 2 * W * 16;                                               // [W]
  int* scl = (int*)(sxp + W);                                                   // [CW][2] block scale exponents
  uint32_t* idx_all = (uint32_t*)(smem + K::kTableBytes + K::kRedBytes);       // [W][16][S]
  unsigned char* bstage_all = smem + K::kTableBytes + K::kRedBytes + K::kIdxBytes;  // [CW][NSET][2048]; wide: [W][2048]
  uint16_t* xf = (uint16_t*)(smem + K::kTableBytes + K::kRedBytes + K::kWorkBytes);   // FUSED: [kXfElems]

  const int tid = threadIdx.x, lane = tid & 63;
  STAMP(0);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cw = wave & (CW - 1), team = wave / CW;          // column wave, team
  const int r = lane & 15, q = lane >> 4;
  // this workgroup's matrix, and its number among the workgroups of that matrix
  // No division, and the pointers and row counts of all four matrices are fetched from the kernel arguments at fixed
  // offsets and then selected: indexed by `mat` they would be fetched only after `mat` is known -- three dependent
  // trips to memory before the first vector load instead of one.  (The empty statement pins all fetches in front of
  // the selection; left alone, the compiler moves each one under a branch on `mat`, behind the wait for `first`.)
  int f1 = mm.first[1], f2 = mm.first[2], f3 = mm.first[3], f4 = mm.first[4];
  int o0 = mm.out[0], o1 = mm.out[1], o2 = mm.out[2], o3 = mm.out[3];
  const uint32_t *pk0 = mm.packed[0], *pk1 = mm.packed[1], *pk2 = mm.packed[2], *pk3 = mm.packed[3];
  const uint32_t *cb0 = mm.codebook[0], *cb1 = mm.codebook[1], *cb2 = mm.codebook[2], *cb3 = mm.codebook[3];
  const float *al0 = mm.alpha[0], *al1 = mm.alpha[1], *al2 = mm.alpha[2], *al3 = mm.alpha[3];
  const float *mu0 = mm.mu[0], *mu1 = mm.mu[1], *mu2 = mm.mu[2], *mu3 = mm.mu[3];
  Dims d = d_arg;
  const __half* x = x_arg;
  int x_dword = x_dword_arg;
  asm volatile("" : "+s"(f1), "+s"(f2), "+s"(f3), "+s"(f4), "+s"(o0), "+s"(o1), "+s"(o2), "+s"(o3),
                    "+s"(pk0), "+s"(pk1), "+s"(pk2), "+s"(pk3), "+s"(cb0), "+s"(cb1), "+s"(cb2), "+s"(cb3),
                    "+s"(al0), "+s"(al1), "+s"(al2), "+s"(al3), "+s"(mu0), "+s"(mu1), "+s"(mu2), "+s"(mu3),
                    "+s"(x), "+s"(x_dword), "+s"(d.in), "+s"(d.wpr));
  const int bx = (int)blockIdx.x;
  const int mat = (bx >= f1 ? 1 : 0) + (bx >= f2 ? 1 : 0) + (bx >= f3 ? 1 : 0);
  auto pick = [mat](auto a0, auto a1, auto a2, auto a3) { return mat == 0 ? a0 : mat == 1 ? a1 : mat == 2 ? a2 : a3; };
  const int wg_first = pick(0, f1, f2, f3);
  const int bid = bx - wg_first;
  const int stride = pick(f1, f2, f3, f4) - wg_first;        // workgroups of this matrix = row blocks between
                                                             // successive ones of a team slot
  d.out = pick(o0, o1, o2, o3);
  const int n_rb = (d.out + 15) >> 4;
  // (behind the empty statement the compiler no longer knows that these point to global memory: said again)
  typedef const __attribute__((address_space(1))) uint32_t* gu32;
  typedef const __attribute__((address_space(1))) float* gf32;
  const uint32_t* __restrict__ packed = pick(pk0, pk1, pk2, pk3);
  const gu32 codebook = (gu32)pick(cb0, cb1, cb2, cb3);

  // ---- small loads first (their data is needed first): codewords, then this wave's share of the activations.
  // An item is 16 consecutive B bytes of one step: (step t, strand qa, half h) = slots e = 16 h .. 16 h + 15
  // of strand qa.  Slot k = 32 qa + e of an instruction sits in B lane k block q' = 2 (qa & 1) + (e >> 4) at
  // byte 16 (qa >> 1) + (e & 15).  The two teams share the B operands: team h prepares the items of half h.
  // FUSED: the waves that own a stage-1 tile of the transform leave the table to the others, so that their
  // matrix-core work overlaps the table build instead of following it.
  constexpr int TW0 = FUSED ? FT_NT : 0;                     // first wave that builds the table
  constexpr int TT = (W - TW0) * 64;                         // threads that build it
  constexpr int KPT = ((1 << B) + TT - 1) / TT;
  const int ttid = tid - TW0 * 64;                           // this thread's number among them (negative: not one)
  uint32_t cwd[KPT];
#pragma unroll
  for (int i = 0; i < KPT; ++i) cwd[i] = codebook[min(max(ttid, 0) + i * TT, (1 << B) - 1)];
  unsigned char* bstage = WIDE ? (unsigned char*)(idx_all + wave * (16 * S)) : bstage_all + cw * (K::NSET * kSetBytes);
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, d.in * 2, kRsrcFlags);
  // With two teams, team e prepares the steps t = e, e + 2, ...: a step's B operand then carries one block
  // scale, and steps of different parity never share an accumulator.
  // SOLO: with at most eight steps the items of BOTH teams fit one wave (8 T <= 64 lanes), so team 0 prepares all B
  // operands of its column wave, under one block scale, and the waves of team 1 skip the conversion: half as many
  // prologue instructions on every SIMD (with three steps per team only 24 of a wave's 64 lanes had an item).
  constexpr bool SOLO = !WIDE && TEAMS == 2 && 8 * T <= 64;
  constexpr bool SPLIT = TEAMS == 2 && !SOLO;               // the teams prepare the steps of one parity each
  const bool prep = !SOLO || team == 0;                     // (wave-uniform) this wave prepares B operands
  constexpr int n_items = WIDE ? 0 : 8 * (SPLIT ? (T + 1) / 2 : T);
  constexpr int NI = WIDE ? 1 : (n_items + 63) / 64;
  uint32_t hx[NI][8];                                      // 16 fp16 values per item, in slot order
  // wide: one half item (8 slots) per lane and set: step 4 tt + lane / 16, strand (lane / 4) % 4, half (lane / 2) % 2,
  // quarter lane % 2 -- chunk 0, chunk 1, chunk 2 (elements 0..7 each) or the three tails
  uint32_t hw[WIDE ? K::NSET : 1][4];
  // 16 or 4 bytes of the activation row at a byte offset (a multiple of 4), zeros when !ok or past the end of the
  // row: from global memory, or (FUSED) from the transformed row in LDS, which holds zeros past the end
  auto xl128 = [&](bool ok, uint32_t off) __attribute__((always_inline)) -> u32x4 {
    if constexpr (FUSED) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (ok) {
        const uint32_t* p = (const uint32_t*)((const unsigned char*)xf + off);
        v = u32x4{p[0], p[1], p[2], p[3]};
      }
      return v;
    } else {
      const auto t4 = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? off : kOob, 0, 0);
      return u32x4{t4[0], t4[1], t4[2], t4[3]};
    }
  };
  auto xl32 = [&](bool ok, uint32_t off) __attribute__((always_inline)) -> uint32_t {
    if constexpr (FUSED) return ok ? *(const uint32_t*)((const unsigned char*)xf + off) : 0u;
    else return __builtin_amdgcn_raw_buffer_load_b32(rx, ok ? off : kOob, 0, 0);
  };
  // The loads of the aligned path (x_dword) are only issued by load_items; merge_items, called where the
  // values are first needed, puts them together.  Every load of the prologue -- codewords, activations, first
  // index words -- is then in flight before the first wait (merged on the spot, the activations cost a trip
  // to memory of their own before the index words were even requested).
  constexpr int NRAW = WIDE ? K::NSET : NI;
  u32x4 raw_a[NRAW], raw_b[WIDE ? 1 : NI];
  uint32_t raw_t[NRAW][3];
  auto load_items = [&]() __attribute__((always_inline)) {
  if constexpr (WIDE) {
    if (x_dword) {
#pragma unroll
      for (int tt = 0; tt < K::NSET; ++tt) {
        const int t = 4 * tt + (lane >> 4), qa = (lane >> 2) & 3, part = lane & 3;
        const uint32_t xb = (uint32_t)((cw * 4 + qa) * L + G * t) * V;
        const bool live = t < T;
        raw_a[tt] = xl128(live && part < 3, (xb + part * V) * 2u);
#pragma unroll
        for (int c = 0; c < 3; ++c)
          raw_t[tt][c] = TAIL == 2 ? xl32(live && part == 3, (xb + c * V + 8u) * 2u) : 0u;
      }
    } else {
#pragma unroll
      for (int tt = 0; tt < K::NSET; ++tt) {
        const int t = 4 * tt + (lane >> 4), qa = (lane >> 2) & 3, part = lane & 3;
        const uint32_t xb = (uint32_t)((cw * 4 + qa) * L + G * t) * V;
        const bool live = t < T;
        uint32_t hv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const bool pad = part == 3 && e >= 3 * TAIL;
          const uint32_t xe = part < 3 ? xb + part * V + e : xb + (uint32_t)(e / TAIL) * V + 8u + (uint32_t)(e % TAIL);
          hv[e] = __builtin_amdgcn_raw_buffer_load_b16(rx, (live && !pad) ? xe * 2u : kOob, 0, 0) & 0xFFFFu;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) hw[tt][k] = hv[2 * k] | (hv[2 * k + 1] << 16);
      }
    }
  }
#pragma unroll
  for (int ii = 0; ii < (WIDE ? 0 : NI); ++ii) {
    const int item = lane + 64 * ii;
    const int t = SPLIT ? 2 * (item >> 3) + team : item >> 3;
    const int qa = (item >> 1) & 3;
    const int h = item & 1;
    const uint32_t xb = (uint32_t)((cw * 4 + qa) * L + G * t) * V;   // first element of the step's three chunks
    const bool live = t < T;
    // half 0: chunk 0 elements 0..7, chunk 1 elements 0..7; half 1: chunk 2 elements 0..7, then the tails
    const uint32_t run0 = h == 0 ? xb : xb + 2u * V;
    if (x_dword) {        // V and `in` even: every pair of elements is one aligned word
      raw_a[ii] = xl128(live, run0 * 2u);
      raw_b[ii] = xl128(live && h == 0, (xb + V) * 2u);
#pragma unroll
      for (int c = 0; c < 3; ++c)
        raw_t[ii][c] = TAIL == 2 ? xl32(live && h == 1, (xb + c * V + 8u) * 2u) : 0u;
    } else {
      uint32_t hv[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        // element of x in slot 16 h + e
        uint32_t xe;
        bool pad = false;
        if (e < 8) xe = run0 + e;
        else if (h == 0) xe = xb + V + (e - 8);
        else {
          const int k = e - 8;                 // tail slot
          pad = k >= 3 * TAIL;
          xe = xb + (uint32_t)(k / TAIL) * V + 8u + (uint32_t)(k % TAIL);
        }
        hv[e] = __builtin_amdgcn_raw_buffer_load_b16(rx, (live && !pad) ? xe * 2u : kOob, 0, 0) & 0xFFFFu;
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) hx[ii][k] = hv[2 * k] | (hv[2 * k + 1] << 16);
    }
  }

  };   // load_items
  // (out-of-range loads return zeros: a lane has either the second 16 bytes or the tails, never both)
  auto merge_items = [&]() __attribute__((always_inline)) {
    if (!x_dword) return;
    if constexpr (WIDE) {
#pragma unroll
      for (int tt = 0; tt < K::NSET; ++tt) {
        hw[tt][0] = raw_a[tt][0] | raw_t[tt][0];
        hw[tt][1] = raw_a[tt][1] | raw_t[tt][1];
        hw[tt][2] = raw_a[tt][2] | raw_t[tt][2];
        hw[tt][3] = raw_a[tt][3];
      }
    } else {
#pragma unroll
      for (int ii = 0; ii < NI; ++ii) {
#pragma unroll
        for (int k = 0; k < 4; ++k) hx[ii][k] = raw_a[ii][k];
        hx[ii][4] = raw_b[ii][0] | raw_t[ii][0];
        hx[ii][5] = raw_b[ii][1] | raw_t[ii][1];
        hx[ii][6] = raw_b[ii][2] | raw_t[ii][2];
        hx[ii][7] = raw_b[ii][3];
      }
    }
  };
  if constexpr (!FUSED) {
    if (prep) load_items();
  }

  // ---- index words.  The wave's four strands are one contiguous piece of every row: LPR lanes fetch it as
  // 16-byte pieces (neighbouring lanes read neighbouring addresses), RPI rows per instruction; the pieces go
  // through a wave-private LDS area from which lane (row r, strand q) reads its own run of words.
  const uint32_t wbit0 = (uint32_t)(cw * 4 * L) * B;         // first bit of the wave's piece inside a row
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
  uint32_t* idx_stage = idx_all + wave * (16 * S);
  auto stage_block = [&](const uint4 (&src)[NLD]) {
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      const int rr = j * RPI + lrow;
      if (lrow < RPI && rr < 16) *(uint4*)(idx_stage + rr * S + 4 * lpc) = src[j];
    }
  };
  // this wave's row blocks: bid + (TEAMS * i + team) * stride, i = 0, 1, ...
  const int rb_first = bid + team * stride, rb_step = TEAMS * stride;
  // Only the first row block is requested now: all waves of all workgroups get their first words within the
  // first burst, instead of queueing behind the later row blocks of the waves that happened to issue first.
  uint4 D0[NLD];
  load_block(rb_first, D0);
  // the operands of the transform are requested after the first index words: they queue behind them in the
  // memory pipeline of the compute unit and are needed later
  typename FT::Ring ring;
  if constexpr (FUSED) FT::begin(geo, (const uint16_t*)x_arg, tid, wave, lane, ring);   // (the argument itself: known to be global memory)
  // (selected only now: the row loop is their first user, and the loads above are not kept waiting for them)
  const gf32 alpha = (gf32)pick(al0, al1, al2, al3);
  const gf32 mu = (gf32)pick(mu0, mu1, mu2, mu3);
  void* const y = pick(mm.y[0], mm.y[1], mm.y[2], mm.y[3]);
  STAMP(1);

  // ---- codebook -> table of nibble patterns, every entry C times, two copies per 16-byte write.  Thread k writes
  // its entry's pairs of copies in the order k, k + 1, ... (mod C / 2): at every step the 16 threads of consecutive
  // entries write 16 different groups of four banks, although an entry's copies are 128 bytes or more apart from
  // the next entry's.
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    const int k = ttid + i * TT;
    if (ttid >= 0 && k < (1 << B)) {
      const unsigned long long ent = expand_codeword<V>(cwd[i]);
      const u32x4 two = {(uint32_t)ent, (uint32_t)(ent >> 32), (uint32_t)ent, (uint32_t)(ent >> 32)};
      u32x4* const row = (u32x4*)(table + k * C);
#pragma unroll
      for (int c = 0; c < C / 2; ++c) row[(c + k) & (C / 2 - 1)] = two;
    }
  }
  STAMP(2);

  if constexpr (FUSED) {
    // the transformed row: zeros past its end, the row itself by the matrix cores; the tiles of the intermediate
    // pass through the index and staging areas, which nothing has used yet
    for (int i = d.in + tid; i < K::kXfElems; i += W * 64) xf[i] = 0;
    static_assert(!FUSED || 2 * FT::NT <= W, "a wave per tile and stage");
    FT::transform_row(tid, wave, lane, ring, xf, (ftr::u32x4*)idx_all);
    STAMP(3);
    __syncthreads();
    STAMP(4);
    if (geo.xt_out != nullptr && blockIdx.x == 0)      // the row for other consumers of the same transform
      for (int i = tid; i < d.in / 2; i += W * 64) ((uint32_t*)geo.xt_out)[i] = ((const uint32_t*)xf)[i];
    if (prep) load_items();
    __syncthreads();   // the exchange area becomes the staging area again
    STAMP(60);
  }
  if (!WIDE && (T & 3)) {   // B columns of steps that do not exist must not hold junk (the two teams share the clearing)
    uint4* z = (uint4*)(bstage + (K::NSET - 1) * kSetBytes + (T & 3) * 512) + team * ((4 - (T & 3)) * 32 / TEAMS);
    for (int i = lane; i < (4 - (T & 3)) * 32 / TEAMS; i += 64) z[i] = make_uint4(0, 0, 0, 0);
  }
  // ---- activations -> four E5M2 pieces each (the top byte of an fp16 IS an E5M2 number; subtracting it
  // leaves at most 8 significant bits, exactly), written in B-operand layout: 16 bytes per item and piece
  // Block scale: 2^k brings the largest element this wave stages to 2^14..2^15 (positive fp16 bit patterns
  // order like integers); the B lanes that hold this wave's items hand 2^-k to the matrix instruction.
  if (prep) merge_items();
  float sx_lane = 0.f;
  int k_scale = 0;
  if (prep) {
    // largest magnitude of this lane's items: packed fp16 maximum of the absolute values, then the two halves
    f16x2 m2 = {(_Float16)0.0f, (_Float16)0.0f};
#pragma unroll
    for (int ii = 0; ii < (WIDE ? 0 : NI); ++ii)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(f16x2, hx[ii][i] & 0x7FFF7FFFu));
    if constexpr (WIDE) {
#pragma unroll
      for (int tt = 0; tt < K::NSET; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(f16x2, hw[tt][i] & 0x7FFF7FFFu));
    }
    const uint32_t mb = __builtin_bit_cast(uint32_t, m2);
    uint32_t mx = max(mb & 0xFFFFu, mb >> 16);
    mx = __builtin_amdgcn_readlane((int)wave_max_to_lane63(mx), 63);
    const int e_field = (int)(mx >> 10);                 // 0 for subnormals, 31 for infinities and NaNs
    k_scale = 29 - max(e_field, 1);
    if (lane == 0) {
      if (SPLIT) scl[cw * 2 + team] = k_scale;
      else scl[cw * 2] = scl[cw * 2 + 1] = k_scale;
    }
  }
  i32x8 Bq[K::NSET];       // B operands: lane (column n = r, k block q) of set tt holds piece n % 4 of step 4 tt + n / 4
  if constexpr (WIDE) {
    // one set at a time through this wave's 2 KB buffer: 64 half items of 8 slots, then every lane reads its 32 bytes
    const int qa = (lane >> 2) & 3, part = lane & 3;
    unsigned char* dst = bstage + (lane >> 4) * 512 + (2 * (qa & 1) + (part >> 1)) * 32 + 16 * (qa >> 1) + 8 * (part & 1);
    const int m1 = k_scale > 15 ? 15 : k_scale;
    const uint32_t pw1 = (uint32_t)(15 + m1) << 10, pw2 = (uint32_t)(15 + (k_scale > 15 ? k_scale - 15 : 0)) << 10;
    const f16x2 f1 = __builtin_bit_cast(f16x2, pw1 | (pw1 << 16)), f2 = __builtin_bit_cast(f16x2, pw2 | (pw2 << 16));
#pragma unroll
    for (int tt = 0; tt < K::NSET; ++tt) {
      uint32_t res[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
        sx_lane = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, hw[tt][i]), one, sx_lane, false);
        res[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, hw[tt][i]) * f1 * f2);   // x * 2^k, exactly
      }
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const uint32_t o0 = __builtin_amdgcn_perm(res[1], res[0], 0x07050301u);
        const uint32_t o1 = __builtin_amdgcn_perm(res[3], res[2], 0x07050301u);
        *(uint2*)(dst + n * 128) = make_uint2(o0, o1);     // steps past T stage zeros (their loads returned zeros)
        if (n < 3) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const f16x2 top = __builtin_bit_cast(f16x2, res[i] & 0xFF00FF00u);
            res[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, res[i]) - top);
          }
        }
      }
      wave_lds_order();
      const uint4* src = (const uint4*)(bstage + r * 128 + q * 32);
      const uint4 lo = src[0], hi = src[1];
      Bq[tt] = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
      wave_lds_order();
    }
  }
  if (prep) {
#pragma unroll
  for (int ii = 0; ii < (WIDE ? 0 : NI); ++ii) {
    const int item = lane + 64 * ii;
    const int t = SPLIT ? 2 * (item >> 3) + team : item >> 3;
    const int qa = (item >> 1) & 3;
    const int h = item & 1;
    // piece n of step t is column 4 (t % 4) + n of set t / 4
    unsigned char* dst = bstage + (t >> 2) * kSetBytes + (t & 3) * 512 + (2 * (qa & 1) + h) * 32 + 16 * (qa >> 1);
    uint32_t res[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      res[i] = hx[ii][i];
      const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
      sx_lane = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, res[i]), one, sx_lane, false);
    }
    // x * 2^k, exactly (k is the same for the whole wave): one multiplication by at most 2^15, and a second
    // one when the whole block is below 2^-1
    {
      const int m = k_scale > 15 ? 15 : k_scale;
      const uint32_t pw = (uint32_t)(15 + m) << 10;
      const f16x2 f = __builtin_bit_cast(f16x2, pw | (pw << 16));
#pragma unroll
      for (int i = 0; i < 8; ++i) res[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, res[i]) * f);
      if (k_scale > 15) {
        const uint32_t pw2 = (uint32_t)(15 + (k_scale - 15)) << 10;
        const f16x2 f2 = __builtin_bit_cast(f16x2, pw2 | (pw2 << 16));
#pragma unroll
        for (int i = 0; i < 8; ++i) res[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, res[i]) * f2);
      }
    }
    if (t < T) {
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        uint32_t o4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)   // bytes 1 and 3 of two dwords: the pieces of four consecutive slots
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
  }   // prep
  STAMP(5);
  // sum of this wave's share of the activations (every element belongs to exactly one item)
  sx_lane = wave_sum_to_lane63(sx_lane);
  if (lane == 63) sxp[wave] = sx_lane;
  // the next row blocks are requested, the first one's index words go to LDS
#pragma unroll
  for (int u = 0; u < kPD; ++u) load_block(rb_first + (u + 1) * rb_step, D[u]);
  stage_block(D0);
  STAMP(6);
  __syncthreads();   // table complete, B operands staged, sums of x stored
  STAMP(7);
  float sx = 0.f;
  static_assert(W % 4 == 0 && (K::kTableBytes + 2 * W * 16 * 4) % 16 == 0, "the wave sums are read four at a time");
#pragma unroll
  for (int w = 0; w < W; w += 4) {   // (same order of additions in every wave)
    const float4 v = *(const float4*)(sxp + w);
    sx += v.x;
    sx += v.y;
    sx += v.z;
    sx += v.w;
  }

  // ---- per-lane constants of the read-back: lane (r, q) starts at bit ws0 + q L B of its staged row
  const uint32_t lbit = (wbit0 & 31u) + (uint32_t)(q * L) * B;
  const uint32_t s0 = lbit & 31u;
  const uint32_t* my_words = idx_stage + r * S + (lbit >> 5);
  const uint32_t lane_copy = (uint32_t)(lane & (C - 1)) * 8u;   // this lane's copy of every table entry
  // inverse block scale of the accumulator class this lane keeps (class c = column / 4 collects the steps
  // t = c mod 4, prepared by team c mod 2)
  const float my_scale = __builtin_ldexpf(1.0f, -scl[cw * 2 + ((r >> 2) & 1)]);
  // the shared B operands are complete: every wave takes its registers
#pragma unroll
  for (int tt = 0; tt < (WIDE ? 0 : K::NSET); ++tt) {
    const uint4* src = (const uint4*)(bstage + tt * kSetBytes + r * 128 + q * 32);
    const uint4 lo = src[0], hi = src[1];
    Bq[tt] = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
  }

  int it = 0;
  for (int rb0 = rb_first; rb0 < n_rb + (TEAMS - 1) * stride; rb0 += kPD * rb_step) {
#pragma unroll
    for (int u = 0; u < kPD; ++u) {
      const int rb = rb0 + u * rb_step;                      // may be past the end (second team): zeros, not stored
      if (rb - team * stride >= n_rb) break;                 // the same for both teams: they share the barriers
      // the wave that will finish this row block asks for its scales now
      const int fw = (it + team * (W / 2 + 1)) % W;          // rotates; the two teams' finishers differ
      const int my_row = rb * 16 + lane;
      const bool finishes = wave == fw && lane < 16 && rb < n_rb && my_row < d.out;
      float al = 0.f, mm = 0.f;
      if (finishes) {
        al = alpha[my_row];
        mm = mu[my_row];
      }
      // this row block's words from LDS; then the next one's take their place (LDS operations of a wave
      // complete in order) and the registers are refilled with the one after those in flight
      wave_lds_order();
      uint32_t Wd[ND + 1];
#pragma unroll
      for (int i = 0; i <= ND; ++i) Wd[i] = my_words[i];
      wave_lds_order();
      stage_block(D[u]);
      load_block(rb + (kPD + 1) * rb_step, D[u]);
      uint32_t R[ND];     // normalised: bit 0 is the first bit of the lane's run
#pragma unroll
      for (int i = 0; i < ND; ++i) R[i] = __builtin_amdgcn_alignbit(Wd[i + 1], Wd[i], s0);
      if (it < 8) STAMP(8 + 5 * it);

      // The step loop, software-pipelined by hand: the LDS reads of step t + 1 (three table entries, the
      // B operand) are issued before the entries of step t are merged and contracted, so an LDS round trip
      // is covered by a step's worth of arithmetic.  (Left to itself the compiler waits for every read.)
      f32x4 acc[4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
      // a table entry as two separate words (as one 64-bit integer the compiler turns "high word << 8" into a
      // funnel shift of both words plus a mask)
      u32x2 E[2][G];   // [pipeline stage][chunk]
      auto issue = [&](int t, u32x2 (&dst)[G]) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const int pos = (t * G + g) * B, w = pos >> 5, sb = pos & 31;
          uint32_t ofs;
          if (B == 8 && C == 32) {
            // byte-aligned indices, 32 copies: offset = index << 8 | copy, assembled by one byte permute
            ofs = __builtin_amdgcn_perm(R[w], lane_copy, 0x0C0C0000u | ((4u + (sb >> 3)) << 8));
          } else {
            // table offset of the entry = index << SH | copy: the field is extracted already shifted
            constexpr int SH = 3 + K::LOG2C;
            constexpr uint32_t mask = ((1u << B) - 1u) << SH;
            uint32_t sh;
            if (sb + B <= 32) sh = sb >= SH ? R[w] >> (sb - SH) : R[w] << (SH - sb);
            else sh = sb >= SH ? __builtin_amdgcn_alignbit(R[w + 1], R[w], sb - SH)
                               : __builtin_amdgcn_alignbit(R[w + 1], R[w], sb) << SH;
            ofs = (sh & mask) | lane_copy;
          }
          // the table starts at LDS address 0 (this kernel has no static LDS), so the offset IS the address
          dst[g] = *(const lds_u32x2*)(uintptr_t)ofs;
        }
      };
      auto consume = [&](int t, const u32x2 (&src)[G]) {
        // two shift-and-or instructions (the byte permute keeps the compiler from re-associating them into two
        // shifts and a three-way or)
        uint32_t tails;
        if constexpr (TAIL == 2) {
          const uint32_t t01 = __builtin_amdgcn_perm(src[1].y, src[0].y, 0x0C0C0400u);   // bytes: t0, t1, 0, 0
          tails = __builtin_amdgcn_perm(src[2].y, t01, 0x0C040100u);                     // bytes: t0, t1, t2, 0
        } else {
          tails = src[0].y | (src[1].y << (4 * TAIL)) | (src[2].y << (8 * TAIL));
        }
        const i32x8 Av = {(int)src[0].x, (int)src[1].x, (int)src[2].x, (int)tails, 0, 0, 0, 0};
        acc[t & 3] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(Av, Bq[t >> 2], acc[t & 3], 4 /* A: E2M1 */,
                                                                      1 /* B: E5M2 */, 0, 0, 0, 0);
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
      if (it < 8) STAMP(9 + 5 * it);
      // Column n of accumulator c is valid for n / 4 == c; a row's sum is the sum of its 16 valid entries.
      // Register i of a lane belongs to row 4 q + i.  The four registers are reduced over the 16 lanes of a
      // row group together: after two select-and-add steps lane n holds the quad sum of register n % 4,
      // after two rotations by 4 and 8 the sum over all 16 lanes.
      float v4[4];
      {
        const int cls = r >> 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float a01 = cls & 1 ? acc[1][i] : acc[0][i];
          const float a23 = cls & 1 ? acc[3][i] : acc[2][i];
          v4[i] = cls & 2 ? a23 : a01;
        }
      }
      const bool odd = r & 1, up = r & 2;
      const float w01 = (odd ? v4[1] : v4[0]) + dpp_xor1(odd ? v4[0] : v4[1]);
      const float w23 = (odd ? v4[3] : v4[2]) + dpp_xor1(odd ? v4[2] : v4[3]);
      float z = (up ? w23 : w01) + dpp_xor2(up ? w01 : w23);   // quad sum: one class, one block scale
      z *= my_scale;
      z += dpp_ror4(z);
      z += dpp_ror8(z);                                      // lane n: the sum of row 4 q + n % 4
      float* rbuf = red + (it & 1) * (W * 16) + team * (CW * 16);
      if (r < 4) rbuf[cw * 16 + 4 * q + r] = z;
      if (it < 8) STAMP(10 + 5 * it);
      __syncthreads();
      if (it < 8) STAMP(11 + 5 * it);
      if (finishes) {
        float tot = 0.f;
#pragma unroll
        for (int w = 0; w < CW; ++w) tot += rbuf[w * 16 + lane];
        const float res = al * tot + mm * sx;
        if (y_is_f32) ((__attribute__((address_space(1))) float*)y)[my_row] = res;
        else ((__attribute__((address_space(1))) uint16_t*)y)[my_row] = __half_as_ushort(__float2half_rn(res));
      }
      if (it < 8) STAMP(12 + 5 * it);
      ++it;
    }
  }
  STAMP(63);
}

template <int V, int B, int T, int TEAMS, int CW, int GN1, int GN2>
static btc_status launch3(hipStream_t q, const Dims& d, const void* x, int y_is_f32, bool dry, const Extra& ex) {
  using K = Cfg<V, B, T, TEAMS, CW, GN1, GN2>;
  static_assert(K::kLdsBytes <= kLdsMax, "LDS budget");
  if (dry) return BTC_OK;         // only asked whether a kernel exists for this setting
  static bool attr_set = false;   // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemv_fp4_kernel<V, B, T, TEAMS, CW, GN1, GN2>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, K::kLdsBytes) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  // One workgroup per compute unit, TEAMS row blocks at a time; the matrices of a launch share the 256 compute
  // units in proportion to their rows: every matrix starts with one workgroup, and the next workgroup goes to the
  // matrix whose workgroups have the most row blocks to walk (the first of them on a tie), until the compute
  // units are used up or no matrix can use another one.
  Multi mm = ex.multi;
  int nrb[kMaxMulti] = {0, 0, 0, 0}, cap[kMaxMulti] = {0, 0, 0, 0}, wg[kMaxMulti] = {0, 0, 0, 0};
  int used = 0;
  for (int m = 0; m < mm.count; ++m) {
    if (mm.out[m] <= 0) mm.out[m] = d.out;
    nrb[m] = (mm.out[m] + 15) / 16;
    cap[m] = (nrb[m] + TEAMS - 1) / TEAMS;
    wg[m] = 1;
    ++used;
  }
  while (used < 256) {
    int best = -1;
    for (int m = 0; m < mm.count; ++m)
      if (wg[m] < cap[m] && (best < 0 || (long long)nrb[m] * wg[best] > (long long)nrb[best] * wg[m])) best = m;
    if (best < 0) break;
    ++wg[best];
    ++used;
  }
  mm.first[0] = 0;
  for (int m = 0; m < kMaxMulti; ++m) mm.first[m + 1] = mm.first[m] + wg[m];
  const int grid = mm.first[kMaxMulti];
  const int x_dword = (V % 2 == 0) && (d.in % 2 == 0);
  gemv_fp4_kernel<V, B, T, TEAMS, CW, GN1, GN2><<<grid, K::W * 64, K::kLdsBytes, q>>>(
      d, mm, (const __half*)x, y_is_f32, x_dword, ex.geo);
  return launch_status();
}

// Steps per row block: the 4 CW strands of a team must cover the row.  Instantiated for a few step counts; a
// strand that is longer than needed reads zeros for the activations past the end of the row.
constexpr int steps_for_chunks(int nchunks, int cw) {
  const int need = (nchunks + cw * 4 * 3 - 1) / (cw * 4 * 3);
  constexpr int have[] = {3, 4, 5, 6, 8, 9, 10, 12, 15, 16};
  constexpr int have_wide[] = {9, 10, 12, 15, 16};        // 17 steps no longer fit 128 registers
  if (cw == 8) {
    for (int t : have) if (need <= t) return t;
  } else {
    for (int t : have_wide) if (need <= t) return t;
  }
  return 0;
}
static int steps_for(const Dims& d, int cw) { return steps_for_chunks(d.nchunks, cw); }

template <int V, int B>
static btc_status launch2(hipStream_t q, const Dims& d, const void* x, int y_is_f32, bool dry, const Extra& ex) {
  // two teams whenever table, staging areas and B operands of 16 waves fit the LDS
#define BTC_FP4_CASE(TT)                                                                                   \
  case TT:                                                                                                 \
    if constexpr (Cfg<V, B, TT, 2, 8>::kLdsBytes <= kLdsMax)                                               \
      return launch3<V, B, TT, 2, 8, 0, 0>(q, d, x, y_is_f32, dry, ex); \
    else if constexpr (Cfg<V, B, TT, 1, 8>::kLdsBytes <= kLdsMax)                                          \
      return launch3<V, B, TT, 1, 8, 0, 0>(q, d, x, y_is_f32, dry, ex); \
    else                                                                                                   \
      break;
#define BTC_FP4_WIDE(TT)                                                                                   \
  case TT:                                                                                                 \
    if constexpr (Cfg<V, B, TT, 1, 16>::kLdsBytes <= kLdsMax)                                              \
      return launch3<V, B, TT, 1, 16, 0, 0>(q, d, x, y_is_f32, dry, ex); \
    else                                                                                                   \
      break;
  switch (steps_for(d, 8)) {
    BTC_FP4_CASE(3) BTC_FP4_CASE(4) BTC_FP4_CASE(5) BTC_FP4_CASE(6) BTC_FP4_CASE(8) BTC_FP4_CASE(9)
    BTC_FP4_CASE(10) BTC_FP4_CASE(12) BTC_FP4_CASE(15) BTC_FP4_CASE(16)
  }
  switch (steps_for(d, 16)) {      // rows too long for eight column waves (or for their LDS areas)
    BTC_FP4_WIDE(9) BTC_FP4_WIDE(10) BTC_FP4_WIDE(12) BTC_FP4_WIDE(15) BTC_FP4_WIDE(16)
  }
#undef BTC_FP4_CASE
#undef BTC_FP4_WIDE
  return BTC_ERR_UNSUPPORTED;
}

template <int V>
static btc_status launch1(hipStream_t q, const Dims& d, const void* x, int y_is_f32, bool dry, const Extra& ex) {
  switch (d.b) {
    case 7: return launch2<V, 7>(q, d, x, y_is_f32, dry, ex);
    case 8: return launch2<V, 8>(q, d, x, y_is_f32, dry, ex);
    case 9: return launch2<V, 9>(q, d, x, y_is_f32, dry, ex);
    case 10: return launch2<V, 10>(q, d, x, y_is_f32, dry, ex);
  }
  return BTC_ERR_UNSUPPORTED;
}

// The product behind the transform: chunk length 10, the row is the N1 x N2 activation matrix, so the step count is
// a constant too; two teams of eight column waves (16 waves: up to eight tiles per stage).
template <int B, int N1, int N2>
static btc_status launch_fused(hipStream_t q, const Dims& d, const void* x, int y_is_f32, bool dry, const Extra& ex) {
  constexpr int T = steps_for_chunks((N1 * N2 + 9) / 10, 8);
  if constexpr (T > 0 && 2 * ftr::Shared<N1, N2, 1024>::NT <= 16) {
    if constexpr (Cfg<10, B, T, 2, 8, N1, N2>::kLdsBytes <= kLdsMax)
      return launch3<10, B, T, 2, 8, N1, N2>(q, d, x, y_is_f32, dry, ex);
  }
  return BTC_ERR_UNSUPPORTED;
}

template <int N1, int N2>
static btc_status launch_fused_b(hipStream_t q, const Dims& d, const void* x, int y_is_f32, bool dry, const Extra& ex) {
  switch (d.b) {
    case 7: return launch_fused<7, N1, N2>(q, d, x, y_is_f32, dry, ex);
    case 8: return launch_fused<8, N1, N2>(q, d, x, y_is_f32, dry, ex);
    case 9: return launch_fused<9, N1, N2>(q, d, x, y_is_f32, dry, ex);
    case 10: return launch_fused<10, N1, N2>(q, d, x, y_is_f32, dry, ex);
  }
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace fp4

#ifdef BTC_FP4_STAMPS
extern "C" int btc_debug_fp4_stamps(unsigned long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(fp4::g_stamps), sizeof(unsigned long long) * n);
}
#endif

static btc_status fp4_dispatch(hipStream_t q, const Dims& d, const void* x, int y_is_f32, bool dry, const fp4::Extra& ex,
                               bool fused) {
  if (d.v != 9 && d.v != 10) return BTC_ERR_UNSUPPORTED;
  if (d.b < 7 || d.b > 10) return BTC_ERR_UNSUPPORTED;
  if ((long long)d.out * d.wpr * 4 >= (1LL << 31)) return BTC_ERR_UNSUPPORTED;     // 32-bit byte offsets
  if ((long long)d.nchunks * d.v * 2 >= (1LL << 31)) return BTC_ERR_UNSUPPORTED;
  if (fused) {
    // The transformed row is made in LDS first: aligned pairs of activations, and factor sizes with an instantiated
    // kernel (ftr::geometry_ok) -- the pairs whose product is the hidden width of LLaMA-2 7B and 13B.  Larger
    // factors (64 x 128 for 8192; 86 x 128, 108 x 128, 128 x 224 for the intermediate widths) are two to four times
    // the operand traffic and arithmetic per workgroup and no longer fit the registers of a 16-wave workgroup: they
    // cost more inside every workgroup than as a launch of their own.
    const ftr::Geo& g = ex.geo;
    if (d.v != 10 || g.n1 * g.n2 != d.in) return BTC_ERR_UNSUPPORTED;
    if (g.n1 == 64 && g.n2 == 64) return fp4::launch_fused_b<64, 64>(q, d, x, y_is_f32, dry, ex);
    if (g.n1 == 64 && g.n2 == 80) return fp4::launch_fused_b<64, 80>(q, d, x, y_is_f32, dry, ex);
    return BTC_ERR_UNSUPPORTED;
  }
  if (d.v == 9) return fp4::launch1<9>(q, d, x, y_is_f32, dry, ex);
  return fp4::launch1<10>(q, d, x, y_is_f32, dry, ex);
}

static fp4::Extra extra_one(const uint32_t* packed, const uint32_t* codebook, const float* alpha, const float* mu, void* y) {
  fp4::Extra ex{};
  ex.multi.packed[0] = packed;
  ex.multi.codebook[0] = codebook;
  ex.multi.alpha[0] = alpha;
  ex.multi.mu[0] = mu;
  ex.multi.y[0] = y;
  ex.multi.count = 1;
  return ex;
}

bool gemv_fp4_covers(const Dims& d) {
  return fp4_dispatch(nullptr, d, nullptr, 0, /*dry=*/true, extra_one(nullptr, nullptr, nullptr, nullptr, nullptr), false) == BTC_OK;
}

btc_status gemv_fp4(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  return fp4_dispatch(q, d, x, y_is_f32, /*dry=*/false, extra_one(packed, codebook, alpha, mu, y), false);
}

btc_status gemv_fp4_multi(hipStream_t q, const Dims& d, int count, const int* outs, const uint32_t* const* packed,
                          const uint32_t* const* codebook, const float* const* alpha, const float* const* mu,
                          const void* x, void* const* y, int y_is_f32) {
  if (count < 1 || count > fp4::kMaxMulti) return BTC_ERR_UNSUPPORTED;
  fp4::Extra ex{};
  for (int m = 0; m < count; ++m) {
    if (outs) {
      if (outs[m] < 1 || outs[m] > d.out) return BTC_ERR_SHAPE;   // d carries the largest row count of the launch
      ex.multi.out[m] = outs[m];
    }
    ex.multi.packed[m] = packed[m];
    ex.multi.codebook[m] = codebook[m];
    ex.multi.alpha[m] = alpha[m];
    ex.multi.mu[m] = mu[m];
    ex.multi.y[m] = y[m];
  }
  ex.multi.count = count;
  return fp4_dispatch(q, d, x, y_is_f32, /*dry=*/false, ex, false);
}

bool gemv_fp4_fused_covers(const Dims& d, int n1, int n2) {
  fp4::Extra ex = extra_one(nullptr, nullptr, nullptr, nullptr, nullptr);
  ex.geo = ftr::make_geo(nullptr, nullptr, n1, n2);
  return fp4_dispatch(nullptr, d, nullptr, 0, /*dry=*/true, ex, true) == BTC_OK;
}

btc_status gemv_fp4_fused(hipStream_t q, const Dims& d, int count, const uint32_t* const* packed,
                          const uint32_t* const* codebook, const float* const* alpha, const float* const* mu,
                          const void* x, int n1, int n2, const uint32_t* sign_bits, const void* prepared, void* xt_out,
                          void* const* y, int y_is_f32) {
  if (count < 1 || count > fp4::kMaxMulti) return BTC_ERR_UNSUPPORTED;
  fp4::Extra ex{};
  for (int m = 0; m < count; ++m) {
    ex.multi.packed[m] = packed[m];
    ex.multi.codebook[m] = codebook[m];
    ex.multi.alpha[m] = alpha[m];
    ex.multi.mu[m] = mu[m];
    ex.multi.y[m] = y[m];
  }
  ex.multi.count = count;
  ex.geo = ftr::make_geo(sign_bits, prepared, n1, n2);
  ex.geo.xt_out = (uint16_t*)xt_out;
  return fp4_dispatch(q, d, x, y_is_f32, /*dry=*/false, ex, true);
}

}  // namespace btc
