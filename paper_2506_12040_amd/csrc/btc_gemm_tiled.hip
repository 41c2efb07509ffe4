// Tuned prefill product for chunk length 10:  Y[M][out] = X[M][in] . W_hat^T.
//
// At many activation rows the layer is a dense contraction, so the index
// tiles are decoded into +-1 16-bit tiles in LDS (exact in bf16 and fp16) and
// contracted on the matrix cores with fp32 accumulation; alpha and mu are
// applied afterwards in fp32 (Algorithm "Binary Transformation and
// Compression": W_hat = alpha * B_hat + mu).
//
// Roles inside a workgroup (wave specialisation):
//   * 4 contraction waves, stacked along M.  Wave w owns 64 activation rows
//     and all BN = 32 NF weight rows of the workgroup: 2 x NF accumulators
//     of MFMA 32x32x16.  Its A operand (activations) never touches LDS: lane
//     (row, h) loads 16 consecutive elements straight from global memory and
//     uses them as the k-slices {16h..16h+7} and {16h+8..16h+15} of a block of
//     32 columns.  The B operand uses the same permutation of k inside the
//     block, which costs nothing because it is only an LDS address.
//   * 4 decoder waves.  A work item (row, half) turns 8 chunk indices of one
//     weight row into 80 +-1 values of the next k-tile while the contraction
//     waves work on the current one.  Decoding therefore overlaps the MFMAs
//     in hardware (two waves per SIMD), and its cost is paid once per
//     workgroup, not once per contraction wave.
//   * one barrier per k-tile of 160 columns (16 chunks), two tile buffers.
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
constexpr int kCH = 16;                 // chunks per k-tile
constexpr int kKT = kV * kCH;           // 160 columns per k-tile = 5 blocks of 32
constexpr int kRS = kKT + 8;            // LDS row stride in elements: 336 B, an odd multiple of 16 B
constexpr int kBM = 256;                // activation rows per workgroup
constexpr int kMW = 4;                  // contraction waves
constexpr int kDW = 4;                  // decoder waves (8 waves per workgroup: 2 per SIMD, 256 registers each)
constexpr uint32_t kOob = 0x80000000u;  // buffer offset that is always out of range
constexpr int kRsrcFlags = 0x00020000;
constexpr int kAStage = 2 * 32 * 64;     // bytes of a contraction wave's private activation slots in LDS

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

template <int NF, bool BF16>
__global__ __launch_bounds__((kMW + kDW) * 64) void gemm_tiled_kernel(
    Dims d, const uint32_t* __restrict__ packed, const uint32_t* __restrict__ codebook,
    const float* __restrict__ alpha, const float* __restrict__ mu, const uint16_t* __restrict__ X, int M,
    void* __restrict__ Y, int y_dtype, int m_blocks, int n_blocks, int tiles_per_split, float* __restrict__ part,
    float* __restrict__ rpart) {
  constexpr int BN = 32 * NF;
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* S = (uint16_t*)smem;                         // [2][BN][kRS]
  uint32_t* E = (uint32_t*)(S + 2 * BN * kRS);           // [2^b][8]: codeword -> 5 dwords of +-1 pairs

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

  // Codeword table: built by all threads, but only after each role has put its first global
  // loads in flight (the table needs a round trip of its own for the codebook).
  auto build_table = [&]() {
    const uint32_t one2 = BF16 ? 0x3F803F80u : 0x3C003C00u;
    for (int k = tid; k < (1 << d.b); k += (kMW + kDW) * 64) {
      const uint32_t npat = ~codebook[k];
      uint32_t e[5];
#pragma unroll
      for (int p = 0; p < 5; ++p)
        e[p] = one2 | ((npat << (15 - 2 * p)) & 0x8000u) | ((npat << (30 - 2 * p)) & 0x80000000u);
      *(uint4*)(E + 8 * k) = make_uint4(e[0], e[1], e[2], e[3]);
      E[8 * k + 4] = e[4];
    }
    __syncthreads();
  };

  if (wave >= kMW) {
    // =============================== decoder waves ===============================
    const int did = tid - kMW * 64;                      // 0 .. 255
    // Work items (weight row r, half): 8 chunks = 80 values each, 64 NF items per tile;
    // a thread owns items did and did + 256 (the second one only if it exists).
    constexpr int NI = (2 * BN + kDW * 64 - 1) / (kDW * 64);
    const uint32_t pk_bytes = (uint32_t)d.out * (uint32_t)d.wpr * 4u;
    const __amdgpu_buffer_rsrc_t rP = __builtin_amdgcn_make_buffer_rsrc((void*)packed, 0, (int)pk_bytes, kRsrcFlags);
    uint32_t W[NI][4];
    const bool pair_loads = d.b == 8 && (d.wpr & 1) == 0;   // two-word loads stay 8-byte aligned
    // the 8 b-bit fields of an item start at bit (t*16 + half*8) * b of the row: at most 4 words
    auto fetch = [&](int t) {
#pragma unroll
      for (int it = 0; it < NI; ++it) {
        const int item = did + it * kDW * 64;
        const int r = item >> 1, half = item & 1;
        const int n = n0 + r;
        const int w0 = ((t * kCH + half * 8) * d.b) >> 5;
        const bool ok = item < 2 * BN && n < d.out;
        if (pair_loads) {
          // 8-bit indices: the 8 fields of an item are exactly two words, fetched by one load.
          // (Every lane access costs the L1 a cycle, and the L1 access rate bounds this kernel.)
          const uint32_t off = (ok && w0 + 1 < d.wpr) ? ((uint32_t)n * (uint32_t)d.wpr + (uint32_t)w0) * 4u : kOob;
          const uint2 w2 = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(rP, off, 0, 0));
          W[it][0] = w2.x; W[it][1] = w2.y; W[it][2] = 0u; W[it][3] = 0u;
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const uint32_t off = (ok && w0 + u < d.wpr) ? ((uint32_t)n * (uint32_t)d.wpr + (uint32_t)(w0 + u)) * 4u : kOob;
            W[it][u] = __builtin_amdgcn_raw_buffer_load_b32(rP, off, 0, 0);
          }
        }
      }
    };
    fetch(t_begin);
    build_table();
    for (int lt = 0; lt <= nt; ++lt) {
      const int t = t_begin + lt;
      if (lt < nt) {
        uint32_t A[NI][3];
#pragma unroll
        for (int it = 0; it < NI; ++it) {                // align the window to the first field
          const int half = (did + it * kDW * 64) & 1;
          const uint32_t s0 = (uint32_t)((t * kCH + half * 8) * d.b) & 31u;
#pragma unroll
          for (int u = 0; u < 3; ++u) A[it][u] = __builtin_amdgcn_alignbit(W[it][u + 1], W[it][u], s0);
        }
        if (lt + 1 < nt) fetch(t + 1);                   // next tile's words fly while this one is expanded
#pragma unroll
        for (int it = 0; it < NI; ++it) {
          const int item = did + it * kDW * 64;
          if (item < 2 * BN) {
            const int r = item >> 1, half = item & 1;
            const bool row_ok = n0 + r < d.out;
            uint16_t* dst = S + (lt & 1) * (BN * kRS) + r * kRS + half * (8 * kV);
            const int j0 = t * kCH + half * 8;
            const uint32_t mask = (1u << d.b) - 1u;
#pragma unroll
            for (int cs = 0; cs < 8; ++cs) {
              // The lanes of a wave walk their 8 chunks in different rotations: with a common
              // order all rows would hit the same 8 LDS banks (the row stride is a multiple of
              // 16 bytes), rotated they spread over all of them.
              const int c = (cs + r + (r >> 3)) & 7;
              // field c sits at bit c*b of the aligned window (b <= 10: inside 3 words)
              const uint32_t pos = (uint32_t)(c * d.b);
              const uint32_t wlo = pos < 32 ? A[it][0] : (pos < 64 ? A[it][1] : A[it][2]);
              const uint32_t whi = pos < 32 ? A[it][1] : A[it][2];
              const uint32_t code = __builtin_amdgcn_alignbit(whi, wlo, pos & 31u) & mask;
              const bool ok = row_ok && j0 + c < d.nchunks;
              const uint4 e4 = *(const uint4*)(E + 8 * code);
              const uint32_t e5 = E[8 * code + 4];
              uint32_t w[5] = {e4.x, e4.y, e4.z, e4.w, e5};
              if (!ok) {                                 // beyond the matrix: zeros (rare, edge tiles only)
#pragma unroll
                for (int p = 0; p < 5; ++p) w[p] = 0u;
              }
              uint32_t* o = (uint32_t*)(dst + c * kV);   // 20-byte chunks: 4-byte aligned
#pragma unroll
              for (int p = 0; p < 5; ++p) o[p] = w[p];
            }
          }
        }
      }
      __syncthreads();                                   // tile t is complete; tile t-1 has been consumed
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

  // A operand (activations), 64 rows per wave in two fragments of 32.
  // An MFMA lane holds 8 consecutive elements of ONE row, so loading the operand straight from
  // memory makes every lane touch a cache line of its own, and the vector L1 -- about one lane
  // access per cycle -- is what bounds this kernel.  Passing everything through LDS instead
  // trades that for LDS waits of the single contraction wave per SIMD.  So the load is split:
  //   fragment 0 (rows 0..31): lane (row l32, h) reads X[m][k0 + 16 h .. + 15] straight into
  //     registers, three blocks of 32 columns in flight;
  //   fragment 1 (rows 32..63): fetched coalesced -- four consecutive lanes read the 64 bytes a
  //     row has in a block -- parked in a wave-private LDS slot and read back in MFMA layout.
  //     Only this wave touches the slot, so no barrier is involved (LDS operations of a wave
  //     complete in order).  The four 16-byte pieces of a row are stored at position
  //     piece ^ ((row / 2) % 4): the read-back of 8 consecutive rows then hits 8 bank groups.
  const __amdgpu_buffer_rsrc_t rX =
      __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, (int)((long long)M * d.in * 2), kRsrcFlags);
  // Rows m >= M need no test of their own: X is row-major, so they lie past the end of the
  // buffer and the hardware range check returns zeros for them.
  const uint32_t xoff0 = (uint32_t)(((long long)(m0 + wave * 64 + l32) * d.in + 16 * h) * 2);
  const int k_lim = min(d.in, (t_begin + nt) * kKT);     // columns of this workgroup's share end here
  auto load_direct = [&](uint4 (&dst)[2], int k0) {      // k0: first column of a block of 32
    // `in` is a multiple of 16 for this kernel; past the end of the row (or of this workgroup's share of
    // it: those blocks are requested by the pipeline but never used) bit 31 of the offset is set
    const uint32_t past = (uint32_t)(k0 + 16 * h + 16 > k_lim) << 31;
    const uint32_t off = (xoff0 + (uint32_t)k0 * 2u) | past;
    dst[0] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rX, off, 0, 0));
    dst[1] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rX, off + 16u, 0, 0));
  };
  unsigned char* AS = smem + 2 * BN * kRS * 2 + ((size_t)32 << d.b) + wave * kAStage;   // [2][32 rows][64 B]
  const int lrow = lane >> 2, lq = lane & 3;
  const int lpiece = lq ^ ((lrow >> 1) & 3);             // the piece this lane fetches (parked at position lq)
  const uint32_t goff0 = (uint32_t)(((long long)(m0 + wave * 64 + 32 + lrow) * d.in + 8 * lpiece) * 2);
  const uint32_t gstep = (uint32_t)(16LL * d.in * 2);    // load j covers rows 32 + 16 j + lane / 4
  auto load_stage = [&](uint4 (&dst)[2], int k0) {
    const uint32_t past = (uint32_t)(k0 + 8 * lpiece + 8 > k_lim) << 31;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t off = (goff0 + (uint32_t)j * gstep + (uint32_t)k0 * 2u) | past;
      dst[j] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rX, off, 0, 0));
    }
  };
  auto park = [&](int slot, const uint4 (&src)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) *(uint4*)(AS + slot * 2048 + j * 1024 + lane * 16) = src[j];
  };
  const int rsw = (l32 >> 1) & 3;
  const unsigned char* ard0 = AS + l32 * 64 + 16 * ((2 * h) ^ rsw);       // k-slice 0: elements 16 h .. + 7
  const unsigned char* ard1 = AS + l32 * 64 + 16 * ((2 * h + 1) ^ rsw);   // k-slice 1: elements 16 h + 8 .. + 15

  // Software pipeline.  Fragment 0: kAS register slots, a block is requested kAS - 1 blocks
  // before its use (a third slot does not fit the 256 registers next to 160 accumulators and
  // measured no faster when it did).  Fragment 1: two register stages in
  // flight from memory (requested three blocks ahead), two LDS slots (the block in use and the
  // next), two fragment registers (the k-slice in use and the next).  Pattern fragments: one
  // register set; fragment c of the next k-slice is read from LDS right after the two MFMAs
  // that use fragment c of the current slice have been issued.  Slots are compile-time: a tile
  // has 5 blocks, so register slot, LDS slot, stage and tile buffer all follow the parity of the
  // tile's first block: 2 tile bodies.
  constexpr int NB = kKT / 32;                           // blocks per k-tile
  constexpr int kAS = 2;
  uint4 ad[kAS][2];                                      // fragment 0: [slot][k-slice]
  uint4 stg[2][2];                                       // fragment 1: [stage][load]
  uint4 afr[2];                                          // fragment 1: [k-slice]
  uint4 bfr[NF];
  float rsum0 = 0.f;                                     // row l32, this lane's half of the columns
  float rs2[2] = {0.f, 0.f};                             // row 32 + 16 j + lane / 4, this lane's piece
  const int kb = t_begin * kKT;                          // first column of this workgroup's share
#pragma unroll
  for (int i = 0; i < kAS; ++i) load_direct(ad[i], kb + 32 * i);
  load_stage(stg[0], kb);
  load_stage(stg[1], kb + 32);
  build_table();
  auto add_rows2 = [&](const uint4 (&src)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      rs2[j] = pair_sum<BF16>(src[j].x, rs2[j]);
      rs2[j] = pair_sum<BF16>(src[j].y, rs2[j]);
      rs2[j] = pair_sum<BF16>(src[j].z, rs2[j]);
      rs2[j] = pair_sum<BF16>(src[j].w, rs2[j]);
    }
  };
  park(0, stg[0]);
  add_rows2(stg[0]);
  load_stage(stg[0], kb + 64);
  afr[0] = *(const uint4*)ard0;
  __syncthreads();                                       // tile 0 decoded
  const uint16_t* sbase = S + l32 * kRS + 16 * h;
  auto tile = [&](int t, auto variant) {
    constexpr int PAR = decltype(variant)::value & 1;    // tile buffer; parity of the tile's first block
    constexpr int PH = decltype(variant)::value % kAS;   // phase of the register-slot pattern
    const uint16_t* st = sbase + PAR * (BN * kRS);
#pragma unroll
    for (int c = 0; c < NF; ++c) bfr[c] = *(const uint4*)(st + c * 32 * kRS);
#pragma unroll
    for (int T = 0; T < NB; ++T) {
      constexpr int dummy = 0;
      (void)dummy;
      const int aslot = (NB * PH + T) % kAS;
      const int bp = (PAR + T) & 1;                      // parity of this block
      // Fragment 1 of the NEXT block moves from its register stage to the other LDS slot and
      // the stage is refilled with the block three further on.  The scheduler must not move
      // this (or the refills below) to the top of the tile: it would wait there for loads that
      // are meant to stay in flight.
      __builtin_amdgcn_sched_barrier(0);
      park(bp ^ 1, stg[bp ^ 1]);
      add_rows2(stg[bp ^ 1]);                            // (zeros beyond this workgroup's share)
      load_stage(stg[bp ^ 1], t * kKT + (T + 3) * 32);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const int q = 2 * T + s;                         // slice number inside the tile
        if (s == 0) afr[1] = *(const uint4*)(ard1 + bp * 2048);          // next slice: same block
        else afr[0] = *(const uint4*)(ard0 + (bp ^ 1) * 2048);           //   first slice of the next block
#pragma unroll
        for (int c = 0; c < NF; ++c) {
          acc[0][c] = mfma32<BF16>(ad[aslot][s], bfr[c], acc[0][c]);
          acc[1][c] = mfma32<BF16>(afr[s], bfr[c], acc[1][c]);
          if (q + 1 < 2 * NB) bfr[c] = *(const uint4*)(st + c * 32 * kRS + ((q + 1) >> 1) * 32 + 8 * ((q + 1) & 1));
        }
      }
      // row sums of fragment 0 from the block just used, then its slot is refilled
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        rsum0 = pair_sum<BF16>(ad[aslot][s].x, rsum0);
        rsum0 = pair_sum<BF16>(ad[aslot][s].y, rsum0);
        rsum0 = pair_sum<BF16>(ad[aslot][s].z, rsum0);
        rsum0 = pair_sum<BF16>(ad[aslot][s].w, rsum0);
      }
      load_direct(ad[aslot], t * kKT + (T + kAS) * 32);  // kAS blocks ahead (zeros past the end)
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();                                     // tile t consumed; tile t+1 decoded
  };
  for (int lt = 0; lt < nt; lt += 2) {                   // the tile body's variant follows the local tile number
    const int t = t_begin + lt;
    tile(t, std::integral_constant<int, 0>{});
    if (lt + 1 < nt) tile(t + 1, std::integral_constant<int, 1>{});
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
  // row sums: the lanes that shared a row add up (two halves of fragment 0, four pieces of
  // fragment 1), then every lane picks up the 32 sums it needs
  rsum0 += __shfl_xor(rsum0, 32, 64);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    rs2[j] += __shfl_xor(rs2[j], 1, 64);
    rs2[j] += __shfl_xor(rs2[j], 2, 64);
  }
  if (h == 0) {
    rsb[l32] = rsum0;
    const int m = m0 + wave * 64 + l32;
    if (split && m < M) rpart[((size_t)sp * n_blocks + nb) * M + m] = rsum0;
  }
  if (lq == 0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      rsb[32 + 16 * j + lrow] = rs2[j];
      const int m = m0 + wave * 64 + 32 + 16 * j + lrow;
      if (split && m < M) rpart[((size_t)sp * n_blocks + nb) * M + m] = rs2[j];
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
static size_t lds_bytes(int b) { return (size_t)2 * 32 * NF * kRS * 2 + ((size_t)32 << b) + kMW * kAStage; }

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
// all fitted to measurements (microseconds): a k-tile costs 0.15 + 0.17 NF + 0.45 per contraction
// wave that has activation rows (their loads, one L1 access per lane and 16 bytes, bound the
// kernel; the NF term is the decode); prologue and epilogue cost 10 + 2 NF.  Wide tiles win
// unless they leave compute units idle; then the k-tiles of an output tile are dealt to several
// workgroups, which costs a second pass over the partial sums.
static Plan make_plan(const Dims& d, int M) {
  const int m_blocks = (M + kBM - 1) / kBM;
  const int ntiles = (d.nchunks + kCH - 1) / kCH;
  const int waves = (min(M, kBM) + 63) / 64;
  Plan best{5, 1, ntiles, 0.0};
  double best_cost = 1e300;
  for (int nf = 2; nf <= 5; ++nf) {
    const double t_tile = 0.15 + 0.17 * nf + 0.45 * waves;
    const long long tiles_out = (long long)m_blocks * ((d.out + 32 * nf - 1) / (32 * nf));
    for (int sp = 1; sp <= 8; ++sp) {
      const int tps = (ntiles + sp - 1) / sp;
      if (sp > 1 && (tps < 4 || (sp - 1) * tps >= ntiles || M > 65535)) continue;   // short or empty splits; grid limit of the second pass
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
