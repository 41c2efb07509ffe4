// Batch-1 decode product by codebook lookup tables, for index widths 5..10.
//
// Appendix "Binary Codebook LUT-GEMM" turns  y_r = sum_j <x_j, C[I_rj]>  into
// one table lookup and one addition per chunk: CBLUT_j[k] = <x_j, C_k> is
// computed once per chunk column j and gathered by the indices of many rows.
// This kernel keeps that idea and changes how it is carried out on CDNA4:
//
//  * A workgroup (16 waves) owns 64 consecutive chunk columns and R rows, 256 at a time.  Its table
//    T[k][c] = <x_c, C_k> (2^b x 64 fp16 entries) is produced by the matrix
//    cores in one shot -- a (2^b x 16) +-1 matrix times a (16 x 64) block of
//    activations -- instead of the two-stage segment tables of the paper,
//    because MFMA builds 1024 entries per instruction while the vector ALU
//    would need ~5 operations per entry.
//  * Lane l of a wave owns row l of a 64-row tile and walks the 64 columns in
//    the skewed order c = (l + t) mod 64.  At every step the 64 lanes address
//    64 different columns, and the table is laid out so that a column fixes
//    the LDS bank (dword c mod 32 of a 128-byte table row, half c / 32).
//    Random indices therefore never collide on a bank, and every lane
//    accumulates its own row: no cross-lane reduction at all.
//  * The 64 b-bit indices of a row tile (2b words per row) are loaded
//    coalesced, staged through LDS, and read back rotated by l chunks so that
//    step t's index sits at the compile-time bit offset t*b of the lane's
//    registers.
//  * Column blocks are reduced across workgroups through fp32 partials in the
//    workspace; the workgroup of the last column block adds them in a
//    fixed order and applies  y = alpha * d + mu * sum(x)  (dequantisation step
//    of Algorithm "Binary Transformation and Compression").  The result does
//    not depend on arrival order.
//
// A decode call on a 13B-sized matrix lasts a few microseconds, so the serial
// instruction count of a wave matters as much as throughput: global loads go
// through buffer descriptors (hardware range check returns 0 outside the
// matrix or the activation vector, which also realises the zero padding of
// the last chunk), and LDS addresses are one per-lane register plus immediates.
#include <hip/hip_fp16.h>

#include "btc_internal.h"

namespace btc {

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTileCols = 64;   // chunk columns per workgroup
constexpr int kTileRows = 64;   // rows per wave tile
constexpr uint32_t kOob = 0x80000000u;  // buffer offset that is always out of range (buffers are < 2 GiB)
constexpr int kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format

// Workspace carve-up for the table engine (all offsets multiples of 256 bytes).
// sx and partial hold 64-bit slots {fp32 value, tag}: tag 1 = written during
// this call, 0 = empty.  The finalising workgroup empties what it consumes,
// so the whole workspace is zero between calls.
struct LutWorkspace {
  unsigned long long* sx;        // [ceil(out/64)][n_ct]  per-column-block sum of x
  unsigned long long* partial;   // [n_ct][out]           per-column-block row sums
};

static inline size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }

size_t lut_workspace_bytes(const btc_shape& s) {
  const size_t n_ct = (s.nchunks + kTileCols - 1) / kTileCols;
  const size_t n_rt = (s.out + kTileRows - 1) / kTileRows;
  return round256(n_rt * n_ct * 8) + round256(n_ct * (size_t)s.out * 8);
}

size_t gemv_table_region_bytes(const Dims& d) {
  if (!lut_engine_covers(d)) return 256;
  const size_t n_ct = (d.nchunks + kTileCols - 1) / kTileCols;
  const size_t n_rt = (d.out + kTileRows - 1) / kTileRows;
  return round256(n_rt * n_ct * 8) + round256(n_ct * (size_t)d.out * 8);
}

static LutWorkspace carve(void* ws, const Dims& d) {
  const size_t n_ct = (d.nchunks + kTileCols - 1) / kTileCols;
  const size_t n_rt = (d.out + kTileRows - 1) / kTileRows;
  char* p = (char*)ws;
  LutWorkspace w;
  w.sx = (unsigned long long*)p;
  p += round256(n_rt * n_ct * 8);
  w.partial = (unsigned long long*)p;
  return w;
}

__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  const f16x2 h = {(_Float16)lo, (_Float16)hi};
  return __builtin_bit_cast(uint32_t, h);
}

// Agent-scope relaxed accesses: they bypass the caches that are not coherent
// across XCDs, so data written by one workgroup is what another one reads.
__device__ __forceinline__ void store_slot(unsigned long long* p, float v) {
  __hip_atomic_store(p, (1ull << 32) | (unsigned long long)__float_as_uint(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void clear_slot(unsigned long long* p) {
  __hip_atomic_store(p, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_slot(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Value of a slot that another workgroup writes: poll until the tag shows up.
// The bound only guards against a hang if a producer never ran (then NaN).
__device__ __forceinline__ float slot_value(const unsigned long long* p, unsigned long long first) {
  unsigned long long v = first;
  for (int spin = 0; (v >> 32) == 0 && spin < (1 << 22); ++spin) v = load_slot(p);
  return (v >> 32) != 0 ? __uint_as_float((uint32_t)v) : __uint_as_float(0x7FC00000u);
}

// Bits (2i, 2i+1) of n -> two fp16 values, bit set => -1, clear => +1.
__device__ __forceinline__ uint32_t sign_pair(uint32_t n, int i) {
  uint32_t r = 0x3C003C00u;
  r = (r & ~0x8000u) | ((n << (15 - 2 * i)) & 0x8000u);
  r = (r & ~0x80000000u) | ((n << (30 - 2 * i)) & 0x80000000u);
  return r;
}

// Order LDS writes before LDS reads of the SAME wave (different lanes): LDS
// operations of one wave complete in issue order; wait for them and keep the
// compiler from moving accesses across this point.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- pieces of the table build shared by both kernels of this file ------------------------

// Activations of column block ct as MFMA B operands: lane (j = lane % 32, h = lane / 32) gets
// elements 8 h .. 8 h + 7 (and 16 + 8 h .. for chunks longer than 16) of chunk columns j and
// 32 + j.  Elements outside the chunk or past the end of x read as 0, which also realises the
// zero padding of the last chunk.
template <bool WIDE_V, bool X_DWORD>
__device__ __forceinline__ void load_block_activations(const __half* x, const Dims& d, int ct, int j, int h,
                                                       uint4 (&bx)[2][WIDE_V ? 2 : 1]) {
  constexpr int KH = WIDE_V ? 2 : 1;
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, d.in * 2, kRsrcFlags);
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int chunk = ct * kTileCols + nb * 32 + j;
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) {
      const int t0 = kh * 16 + h * 8;
      const uint32_t e0 = (uint32_t)(chunk * d.v + t0) * 2u;   // byte offset of element t0 of the chunk
      uint32_t wv[4];
      if (X_DWORD) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          wv[i] = __builtin_amdgcn_raw_buffer_load_b32(rx, (t0 + 2 * i < d.v) ? e0 + 4u * i : kOob, 0, 0);
      } else {
        uint32_t hv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
          hv[e] = __builtin_amdgcn_raw_buffer_load_b16(rx, (t0 + e < d.v) ? e0 + 2u * e : kOob, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) wv[i] = (hv[2 * i] & 0xFFFFu) | (hv[2 * i + 1] << 16);
      }
      bx[nb][kh] = make_uint4(wv[0], wv[1], wv[2], wv[3]);
    }
  }
}

// Sum of the block's activations over the whole wave (every element is held by exactly one lane).
template <int KH>
__device__ __forceinline__ float block_activation_sum(const uint4 (&bx)[2][KH]) {
  float sxl = 0.f;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) {
      const uint32_t w4[4] = {bx[nb][kh].x, bx[nb][kh].y, bx[nb][kh].z, bx[nb][kh].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const f16x2 p = __builtin_bit_cast(f16x2, w4[i]);
        sxl += (float)p[0];
        sxl += (float)p[1];
      }
    }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sxl += __shfl_xor(sxl, o, 64);
  return sxl;
}

// Table rows of the 32 codewords of group cg: 32 codewords x 64 columns per pair of MFMAs.
// D[i][jj]: lane holds column jj = lane % 32 and codewords i = 8 (e/4) + 4 h + e%4; columns j (low
// half) and 32 + j (high half) of a codeword row share a dword.  npat = ~codeword of lane j.
template <int KH>
__device__ __forceinline__ void build_table_group(uint32_t* table, int cg, uint32_t npat, const uint4 (&bx)[2][KH],
                                                  int j, int h) {
  f32x16 d0, d1;
#pragma unroll
  for (int e = 0; e < 16; ++e) d0[e] = d1[e] = 0.f;
#pragma unroll
  for (int kh = 0; kh < KH; ++kh) {
    const uint32_t n = npat >> (kh * 16 + h * 8);
    const uint4 a = make_uint4(sign_pair(n, 0), sign_pair(n, 1), sign_pair(n, 2), sign_pair(n, 3));
    d0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, bx[0][kh]), d0,
                                                0, 0, 0);
    d1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, bx[1][kh]), d1,
                                                0, 0, 0);
  }
  uint32_t* trow = table + (cg * 32 + 4 * h) * 32 + j;
#pragma unroll
  for (int e = 0; e < 16; ++e) trow[(8 * (e >> 2) + (e & 3)) * 32] = pack_f16x2(d0[e], d1[e]);
}

constexpr int kRowTiles = 4;    // 64-row tiles a workgroup works on at once
constexpr int kQuarters = 4;    // waves that share one row tile: each walks 16 of the 64 columns
constexpr int kWaves = kRowTiles * kQuarters;

template <int B, bool DUP>
struct LutCfg {
  static constexpr int W2 = 2 * B;                       // words per tile row: 64 indices of B bits
  static constexpr int RPI = 64 / W2;                    // tile rows fetched by one wave-wide load
  static constexpr int NQ = (kTileRows + RPI - 1) / RPI; // loads per tile
  static constexpr int NQW = (NQ + kQuarters - 1) / kQuarters;  // loads per tile and wave
  static constexpr int kStageRows = NQW * kQuarters * RPI;      // >= 64
  static constexpr int SR = (DUP ? 2 * W2 : W2) + 1;     // staged row stride in words (odd)
  static constexpr int QW = (16 * B + 31) / 32;          // words holding a quarter's 16 indices
  static constexpr int kTableBytes = (1 << B) * 128;
  static constexpr int kStageBytes = kRowTiles * kStageRows * SR * 4;
  static constexpr int kRedBytes = kWaves * 64 * 4;
  static constexpr int kLdsBytes = kTableBytes + kStageBytes + kRedBytes;
  static constexpr int kGroups = (1 << B) / 32;          // 32-codeword groups
  static constexpr int kGroupsPerWave = (kGroups + kWaves - 1) / kWaves;
};

// Wave w of the 16: row tile w / 4, column quarter w % 4.  The four waves of a row
// tile split everything: the tile's loads, the 64-step walk (16 steps each, which is
// just the original walk started at lane + 16 q) and -- through LDS -- the row sums.
// Spreading a tile over four waves does not change the work, but it shortens the
// serial instruction stream of every wave about fourfold, and at a few microseconds
// per call that stream is what the latency consists of.
template <int B, bool DUP, bool WIDE_V /* v > 16 */, bool X_DWORD /* v and in even */, int D /* tiles in flight */>
__global__ __launch_bounds__(kWaves * 64) void gemv_lut_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                               const uint32_t* __restrict__ codebook,
                                                               const float* __restrict__ alpha,
                                                               const float* __restrict__ mu,
                                                               const __half* __restrict__ x, void* __restrict__ y,
                                                               int y_is_f32, LutWorkspace ws, int n_ct, int n_rb,
                                                               int RT, int fin) {
  using Cfg = LutCfg<B, DUP>;
  constexpr int W2 = Cfg::W2, SR = Cfg::SR, RPI = Cfg::RPI, NQW = Cfg::NQW, QW = Cfg::QW;
  constexpr int KH = WIDE_V ? 2 : 1;
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* table = (uint32_t*)smem;                                   // [2^B][32] dwords of 2 x fp16
  uint32_t* stage_all = (uint32_t*)(smem + Cfg::kTableBytes);
  float* red = (float*)(smem + Cfg::kTableBytes + Cfg::kStageBytes);   // [16 waves][64]

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD whole row
  // blocks so that neighbouring column blocks of a row (which share HBM lines)
  // meet in the same L2.
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int n_cols = n_ct + fin;                         // with fin, workgroup n_ct of a row block only finishes rows
  const int rb = (slot / n_cols) * 8 + xcd;
  const int ct = slot - (slot / n_cols) * n_cols;
  if (rb >= n_rb) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wt = wave >> 2, qw = wave & 3;                             // row tile, column quarter
  // The workgroup of the last column block finishes the rows; it asks for the scale and mean
  // of its first rows now, so that the loads are not a round trip at the end of the call.
  const int rows_per_wg = RT * kRowTiles * kTileRows;
  const int row_first = rb * rows_per_wg + tid;
  float al_first = 0.f, mu_first = 0.f;
  if (D == 1 && ct == n_ct - 1 + fin && tid < 256 && row_first < d.out) {   // the threads that will store the rows
    al_first = alpha[row_first];
    mu_first = mu[row_first];
  }
  // Finishing a row block: add the column blocks' partial sums in order, scale, store (details
  // at the end of the kernel).  Done by the workgroup of the last column block after its own
  // lookups or, with `fin`, by an extra workgroup that does nothing else and therefore polls
  // from the start: the call then ends one poll after the last partial sum lands instead of a
  // production phase plus polls later.  The extra workgroup costs a residency slot, so the host
  // asks for it only when every workgroup of the grid is resident at once anyway.
  const bool finisher = fin && ct == n_ct;
  auto produce = [&]() {
  const int j = lane & 31, h = lane >> 5;
  uint32_t* stage = stage_all + wt * (Cfg::kStageRows * SR);

  // ---- index tiles: lane (lr, lw) fetches word lw of tile rows lr, lr+RPI, ...; the four waves
  // of a row tile take every fourth load
  const int lr = lane / W2, lw = lane - lr * W2;
  const int words_left = d.wpr - ct * W2;                 // words of this column block inside a row
  const bool lane_loads = lr < RPI;
  const uint32_t tile_voff = (lane_loads && lw < words_left) ? (uint32_t)(lr * d.wpr + lw) * 4u : kOob;
  const uint32_t q_stride = (uint32_t)(RPI * d.wpr) * 4u;
  const uint32_t total_bytes = (uint32_t)d.out * (uint32_t)d.wpr * 4u;
  uint32_t ld[D][NQW];
  auto load_tile = [&](int row0, uint32_t (&dst)[NQW]) {
    // descriptor rebased to the tile, so that the range check sees the true distance to the end
    const uint32_t base_off = ((uint32_t)row0 * (uint32_t)d.wpr + (uint32_t)(ct * W2)) * 4u;
    const bool inside = row0 < d.out;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const char*)packed + (inside ? base_off : 0u)), 0, inside ? (int)(total_bytes - base_off) : 0,
        kRsrcFlags);
#pragma unroll
    for (int i = 0; i < NQW; ++i)   // loads q >= NQ fetch rows of the next tile or nothing; they are never used
      dst[i] = __builtin_amdgcn_raw_buffer_load_b32(rs, tile_voff + (uint32_t)(i * kQuarters + qw) * q_stride, 0, 0);
  };
  // The first D tiles are requested before anything else.  HBM latency times bandwidth is
  // several megabytes, so a workgroup that walks many tiles keeps D of them in flight.
  const int first_row = (rb * RT * kRowTiles + wt) * kTileRows;
  constexpr int kStep = kRowTiles * kTileRows;           // rows between successive tiles of a wave
#pragma unroll
  for (int u = 0; u < D; ++u)
    if (u < RT) load_tile(first_row + u * kStep, ld[u]);

  // ---- table build, split over the waves by 32-codeword groups
  const bool builds = wave < Cfg::kGroups;
  uint32_t npat_all[Cfg::kGroupsPerWave];
  uint4 bx[2][KH];
  if (builds) {
#pragma unroll
    for (int it = 0; it < Cfg::kGroupsPerWave; ++it) npat_all[it] = ~codebook[(it * kWaves + wave) * 32 + j];
    load_block_activations<WIDE_V, X_DWORD>(x, d, ct, j, h, bx);
  }

  // ---- per-lane constants of this wave's part of the skewed walk: it starts at virtual
  // lane v0 = lane + 16 q; step i reads column c = (v0 + i) & 63 -> byte offset 4 (c & 31) + 2 (c >> 5)
  const int v0 = (lane + 16 * qw) & 63;
  uint32_t colofs[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const uint32_t c = (uint32_t)(v0 + i);
    colofs[i] = ((c << 2) & 124u) | ((c >> 4) & 2u);
  }
  const int rot_bits = v0 * B;
  const int wr = rot_bits >> 5;
  const uint32_t sh = rot_bits & 31;
  uint32_t* stage_wr = stage + (qw * RPI + lr) * SR + lw;  // where this lane stages what it fetched
  const uint32_t* stage_rd = stage + lane * SR + wr;       // where its quarter of its rotated row starts

  if (builds) {
    if (wave == 0) {  // one wave also adds the block's activations up
      const float sxl = block_activation_sum<KH>(bx);
      if (lane == 0) store_slot(&ws.sx[rb * n_ct + ct], sxl);
    }
#pragma unroll
    for (int it = 0; it < Cfg::kGroupsPerWave; ++it) {
      const int cg = it * kWaves + wave;
      if (cg < Cfg::kGroups) build_table_group<KH>(table, cg, npat_all[it], bx, j, h);
    }
  }

  const char* table_bytes = (const char*)table;
  for (int rt0 = 0; rt0 < RT; rt0 += D) {
#pragma unroll
   for (int u = 0; u < D; ++u) {
    const int rt = rt0 + u;
    if (rt >= RT) break;
    const int row0 = first_row + rt * kStep;
    if (lane_loads) {
#pragma unroll
      for (int i = 0; i < NQW; ++i) {
        stage_wr[i * kQuarters * RPI * SR] = ld[u][i];
        if (DUP) stage_wr[i * kQuarters * RPI * SR + W2] = ld[u][i];
      }
    }
    if (rt + D < RT) load_tile(row0 + D * kStep, ld[u]);  // keeps D tiles in flight
    __syncthreads();  // tile staged by its four waves (first pass: the table is complete, too)
    // read back this wave's quarter, rotated by v0 chunks: R[i] = bits [32 i, 32 i + 32)
    uint32_t Wd[QW + 1];
#pragma unroll
    for (int i = 0; i <= QW; ++i) {
      if (DUP) Wd[i] = stage_rd[i];
      else Wd[i] = stage[lane * SR + (wr + i >= W2 ? wr + i - W2 : wr + i)];
    }
    uint32_t R[QW + 1];
#pragma unroll
    for (int i = 0; i < QW; ++i) R[i] = __builtin_amdgcn_alignbit(Wd[i + 1], Wd[i], sh);
    R[QW] = 0;

    float acc = 0.f;
#pragma unroll
    for (int t = 0; t < 16; t += 2) {
      _Float16 e2[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int p = (t + u) * B, w = p >> 5, s = p & 31;
        uint32_t code;
        if (s + B <= 32) code = (R[w] >> s) & ((1u << B) - 1u);
        else code = __builtin_amdgcn_alignbit(R[w + 1], R[w], s) & ((1u << B) - 1u);
        e2[u] = *(const _Float16*)(table_bytes + ((code << 7) + colofs[t + u]));
      }
      const f16x2 pr = {e2[0], e2[1]};
      const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
      acc = __builtin_amdgcn_fdot2(pr, one, acc, false);
    }
    red[wave * 64 + lane] = acc;
    __syncthreads();  // quarters of a row tile meet; the staging buffers are free again
    if (qw == 0) {
      const float* rp = red + (wt * kQuarters) * 64 + lane;
      const float tot = ((rp[0] + rp[64]) + rp[128]) + rp[192];   // fixed order
      const int row = row0 + lane;
      if (row < d.out) store_slot(&ws.partial[ct * d.out + row], tot);
    }
   }
  }

  // ---- the workgroup of the LAST column block of this row block adds the column blocks
  // in order.  Partials travel as agent-scope (cache-bypassing) 8-byte stores {value, tag}
  // that nobody waits for; the reducing workgroup polls each slot until its tag shows up.
  // Why this cannot hang: producers never wait for anything, and the reducer has the
  // highest workgroup id of its row block (same XCD, ids differ by multiples of 8), so the
  // in-order dispatcher has already placed every producer when the reducer starts.  The
  // poll is bounded all the same; a slot that never arrives yields NaN, not a hang.
  // (An arrival counter would cost a device-scope atomic round trip per workgroup; full
  // agent-scope fences would write back and invalidate the XCD's whole L2, tens of
  // microseconds per workgroup.)
  };
  if (!finisher) {
    produce();
    if (fin || ct != n_ct - 1) return;
  }
  // Four threads share a row: thread (part, r) fetches the column blocks part, part + 4, ... of
  // row r, all in flight at once, and adds them in increasing order; the four sums then meet in
  // LDS and are added in a fixed order too, so the result does not depend on timing.
  float* sx_buf = (float*)stage_all;  // staging space is free now
  float* comb = red;                  // [4][256], free after the last barrier of the main loop
  constexpr int NT = kWaves * 64;
  constexpr int kPB = 12;             // slots per thread and batch: 48 column blocks per batch
  const int part = tid >> 8, rr = tid & 255;
  unsigned long long pb[kPB];
  auto fetch_slots = [&](int row, int c0) {
#pragma unroll
    for (int u = 0; u < kPB; ++u)   // the guard is uniform in a wave (part is), so no lane issues idle loads
      if (c0 + 4 * u < n_ct) pb[u] = load_slot(&ws.partial[(c0 + 4 * u) * d.out + row]);
  };
  auto add_slots = [&](int row, int c0, float acc) {
#pragma unroll
    for (int u = 0; u < kPB; ++u) {
      const int c = c0 + 4 * u;
      if (c < n_ct) {
        unsigned long long* slot = &ws.partial[c * d.out + row];
        acc += slot_value(slot, pb[u]);
        clear_slot(slot);
      }
    }
    return acc;
  };
  if (D == 1) {  // first batch: in flight with the sx loads
    const int row = rb * rows_per_wg + rr;
    if (row < d.out) fetch_slots(row, part);
  }
  // sum of x: every thread adds the column-block sums in the same order
  float sx = 0.f;
  for (int c0 = 0; c0 < n_ct; c0 += NT) {
    __syncthreads();
    if (c0 + tid < n_ct) {
      unsigned long long* slot = &ws.sx[rb * n_ct + c0 + tid];
      sx_buf[tid] = slot_value(slot, load_slot(slot));
      clear_slot(slot);
    }
    __syncthreads();
    const int n = min(NT, n_ct - c0);
    for (int c = 0; c < n; ++c) sx += sx_buf[c];
  }
  if (D == 1) {   // one block of 256 rows per workgroup
    const int row = rb * rows_per_wg + rr;
    const bool ok = row < d.out;
    float dsum = 0.f;
    if (ok) {
      for (int c0 = part; c0 < n_ct; c0 += 4 * kPB) {
        if (c0 != part) fetch_slots(row, c0);
        dsum = add_slots(row, c0, dsum);
      }
    }
    comb[part * 256 + rr] = dsum;
    __syncthreads();
    if (part == 0 && ok) {
      const float tot = ((comb[rr] + comb[256 + rr]) + comb[512 + rr]) + comb[768 + rr];
      const float res = al_first * tot + mu_first * sx;
      if (y_is_f32) ((float*)y)[row] = res;
      else ((__half*)y)[row] = __float2half_rn(res);
    }
  } else {
    // Several row blocks per workgroup: a thread per row keeps more rows in flight at once than
    // four threads per row would, and the rows outnumber the threads anyway.
    for (int r = tid; r < rows_per_wg; r += NT) {
      const int row = rb * rows_per_wg + r;
      if (row >= d.out) break;
      const float al = alpha[row], mm = mu[row];
      float dsum = 0.f;
      for (int c = 0; c < n_ct; c += 16) {
        unsigned long long p16[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) p16[u] = load_slot(&ws.partial[min(c + u, n_ct - 1) * d.out + row]);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          if (c + u < n_ct) {
            unsigned long long* slot = &ws.partial[(c + u) * d.out + row];
            dsum += slot_value(slot, p16[u]);
            clear_slot(slot);
          }
        }
      }
      const float res = al * dsum + mm * sx;
      if (y_is_f32) ((float*)y)[row] = res;
      else ((__half*)y)[row] = __float2half_rn(res);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Streaming variant for matrices of tens of megabytes (used for 9-bit indices).
//
// The kernel above is built for calls that last a few microseconds: it spends instructions
// (a quarter tile per wave, two workgroup barriers per tile) to shorten every wave's serial
// stream.  On a large matrix the same engine is bound by instruction issue, so here the
// trade is reversed: a wave owns a whole 64 x 64 tile (64 lookups per staged tile instead of
// 16, no workgroup barrier after the table is built, wave-private staging), workgroups stay
// resident and build their table once, and each wave keeps two tiles in flight from memory.
// Table, lookup order, partial-sum slots and the finishing workgroup are the same as above.
constexpr int kStreamWaves = 12;

template <int B>
struct StreamCfg {
  static constexpr int W2 = 2 * B;                       // words per tile row: 64 indices of B bits
  static constexpr int RPI = 64 / W2;                    // tile rows fetched by one wave-wide load
  static constexpr int NQ = (kTileRows + RPI - 1) / RPI; // loads per tile
  static constexpr int kStageRows = NQ * RPI;            // >= 64
  static constexpr int SR = W2 + 1;                      // staged row stride in words (odd)
  static constexpr int kTableBytes = (1 << B) * 128;
  static constexpr int kStageBytes = kStreamWaves * kStageRows * SR * 4;
  static constexpr int kLdsBytes = kTableBytes + kStageBytes + 1024;   // + sums of x of the column blocks
  static constexpr int kGroups = (1 << B) / 32;
};

template <int B, bool WIDE_V, bool X_DWORD>
__global__ __launch_bounds__(kStreamWaves * 64) void gemv_lut_stream_kernel(
    Dims d, const uint32_t* __restrict__ packed, const uint32_t* __restrict__ codebook,
    const float* __restrict__ alpha, const float* __restrict__ mu, const __half* __restrict__ x,
    void* __restrict__ y, int y_is_f32, LutWorkspace ws, int n_ct, int n_rb, int tiles_per_wg) {
  using Cfg = StreamCfg<B>;
  constexpr int W2 = Cfg::W2, SR = Cfg::SR, RPI = Cfg::RPI, NQ = Cfg::NQ;
  constexpr int KH = WIDE_V ? 2 : 1;
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* table = (uint32_t*)smem;                                   // [2^B][32] dwords of 2 x fp16
  uint32_t* stage_all = (uint32_t*)(smem + Cfg::kTableBytes);
  float* sx_buf = (float*)(smem + Cfg::kTableBytes + Cfg::kStageBytes);

  // Same XCD-aware numbering as above, with one more workgroup per row block: number n_ct has
  // no column block; it only finishes the rows (below).
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int rb = (slot / (n_ct + 1)) * 8 + xcd;
  const int ct = slot - (slot / (n_ct + 1)) * (n_ct + 1);
  if (rb >= n_rb) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 31, h = lane >> 5;
  uint32_t* stage = stage_all + wave * (Cfg::kStageRows * SR);
  const int tile_first = rb * tiles_per_wg;                            // this workgroup's 64-row tiles
  const int n_tiles_all = (d.out + kTileRows - 1) / kTileRows;
  const int tile_end = min(tile_first + tiles_per_wg, n_tiles_all);

  // ---- index tiles: lane (lr, lw) fetches word lw of tile rows lr, lr + RPI, ...
  const int lr = lane / W2, lw = lane - lr * W2;
  const int words_left = d.wpr - ct * W2;
  const bool lane_loads = lr < RPI;
  const uint32_t tile_voff = (lane_loads && lw < words_left) ? (uint32_t)(lr * d.wpr + lw) * 4u : kOob;
  const uint32_t q_stride = (uint32_t)(RPI * d.wpr) * 4u;
  const uint32_t total_bytes = (uint32_t)d.out * (uint32_t)d.wpr * 4u;
  uint32_t ld[2][NQ];
  auto load_tile = [&](int tile, uint32_t (&dst)[NQ]) {
    const int row0 = tile * kTileRows;
    const bool inside = tile < tile_end;                               // tiles of other workgroups are not fetched
    const uint32_t base_off = inside ? ((uint32_t)row0 * (uint32_t)d.wpr + (uint32_t)(ct * W2)) * 4u : 0u;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const char*)packed + base_off), 0, inside ? (int)(total_bytes - base_off) : 0, kRsrcFlags);
#pragma unroll
    for (int i = 0; i < NQ; ++i) dst[i] = __builtin_amdgcn_raw_buffer_load_b32(rs, tile_voff + (uint32_t)i * q_stride, 0, 0);
  };
  if (ct == n_ct) {
    // ---- The finishing workgroup.  It has the highest workgroup id of its row block, so the
    // in-order dispatcher has placed every producer of the block before it; producers never
    // wait, hence the polls below end (they are bounded all the same: NaN, not a hang).  It
    // starts polling at once and follows the producers tile by tile, so that at the end of
    // the call only the last tiles' round trip is left.
    constexpr int NT = kStreamWaves * 64;
    float sx = 0.f;
    for (int c0 = 0; c0 < n_ct; c0 += 256) {
      __syncthreads();
      if (tid < 256 && c0 + tid < n_ct) {
        unsigned long long* sl = &ws.sx[rb * n_ct + c0 + tid];
        sx_buf[tid] = slot_value(sl, load_slot(sl));
        clear_slot(sl);
      }
      __syncthreads();
      const int n = min(256, n_ct - c0);
      for (int c = 0; c < n; ++c) sx += sx_buf[c];
    }
    const int row_begin = tile_first * kTileRows, row_end = min(tile_end * kTileRows, d.out);
    for (int row = row_begin + tid; row < row_end; row += NT) {
      const float al = alpha[row], mm = mu[row];
      float dsum = 0.f;
      for (int c = 0; c < n_ct; c += 16) {
        unsigned long long p16[16];
#pragma unroll
        for (int u = 0; u < 16; ++u)
          if (c + u < n_ct) p16[u] = load_slot(&ws.partial[(c + u) * d.out + row]);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          if (c + u < n_ct) {
            unsigned long long* sl = &ws.partial[(c + u) * d.out + row];
            dsum += slot_value(sl, p16[u]);
            clear_slot(sl);
          }
        }
      }
      const float res = al * dsum + mm * sx;
      if (y_is_f32) ((float*)y)[row] = res;
      else ((__half*)y)[row] = __float2half_rn(res);
    }
    return;
  }

  // ---- activations first (the table needs them, and loads return in order), then the first
  // two index tiles of this wave; the table build is split over the waves by 32-codeword
  // groups as in the kernel above
  {
    uint4 bx[2][KH];
    if (wave >= Cfg::kGroups) {
      load_tile(tile_first + wave, ld[0]);
    } else {
      load_block_activations<WIDE_V, X_DWORD>(x, d, ct, j, h, bx);
      load_tile(tile_first + wave, ld[0]);   // the second tile is requested after the barrier: issuing it here
                                             // would hold this wave in the (saturated) memory queue while
                                             // the whole workgroup waits for its part of the table
      if (wave == 0) {  // one wave also adds the block's activations up
        const float sxl = block_activation_sum<KH>(bx);
        if (lane == 0) store_slot(&ws.sx[rb * n_ct + ct], sxl);
      }
      for (int cg = wave; cg < Cfg::kGroups; cg += kStreamWaves)
        build_table_group<KH>(table, cg, ~codebook[cg * 32 + j], bx, j, h);
    }
  }

  // ---- per-lane constants of the skewed walk: step i reads column c = (lane + i) & 63
  // (column c + 32 shares the dword of column c and sits in its other half: steps 32..63 reuse
  // the offsets of steps 0..31 with bit 1 flipped, which halves the registers held)
  uint32_t colofs[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const uint32_t c = (uint32_t)(lane + i);
    colofs[i] = ((c << 2) & 124u) | ((c >> 4) & 2u);
  }
  const int rot_bits = lane * B;
  const int wr = rot_bits >> 5;
  const uint32_t sh = rot_bits & 31;
  uint32_t* stage_wr = stage + lr * SR + lw;
  const uint32_t* rd_a = stage + lane * SR + wr;       // word i of the rotated row: rd_a[i], or
  const uint32_t* rd_b = rd_a - W2;                    // rd_b[i] once wr + i has run past the row's end
  __syncthreads();                                     // the table is complete
  load_tile(tile_first + wave + kStreamWaves, ld[1]);

  const char* table_bytes = (const char*)table;
  auto one_tile = [&](int tile, uint32_t (&cur)[NQ]) {
    if (lane_loads) {
#pragma unroll
      for (int i = 0; i < NQ; ++i) stage_wr[i * RPI * SR] = cur[i];
    }
    load_tile(tile + 2 * kStreamWaves, cur);            // two tiles ahead, into the registers just staged
    wave_lds_sync();
    uint32_t Wd[W2];
#pragma unroll
    for (int i = 0; i < W2; ++i) {
      // lanes l >= ceil(32 (W2 - i) / B) have wrapped around at word i
      constexpr int dummy = 0;
      (void)dummy;
      const int first_wrapped = (32 * (W2 - i) + B - 1) / B;
      Wd[i] = (lane >= first_wrapped ? rd_b : rd_a)[i];
    }
    wave_lds_sync();                                    // staging area free for the next tile
    uint32_t R[W2 + 1];
#pragma unroll
    for (int i = 0; i < W2; ++i) R[i] = __builtin_amdgcn_alignbit(Wd[(i + 1) % W2], Wd[i], sh);
    R[W2] = 0;
    float acc = 0.f;
#pragma unroll
    for (int t = 0; t < 64; t += 2) {
      _Float16 e2[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int p = (t + u) * B, w = p >> 5, s = p & 31;
        uint32_t code;
        if (s + B <= 32) code = (R[w] >> s) & ((1u << B) - 1u);
        else code = __builtin_amdgcn_alignbit(R[w + 1], R[w], s) & ((1u << B) - 1u);
        const uint32_t at = (code << 7) | colofs[(t + u) & 31];
        e2[u] = *(const _Float16*)(table_bytes + (t + u < 32 ? at : at ^ 2u));
      }
      const f16x2 pr = {e2[0], e2[1]};
      const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
      acc = __builtin_amdgcn_fdot2(pr, one, acc, false);
    }
    const int row = tile * kTileRows + lane;
    if (row < d.out) store_slot(&ws.partial[ct * d.out + row], acc);
  };
  for (int tile = tile_first + wave; tile < tile_end; tile += 2 * kStreamWaves) {
    one_tile(tile, ld[0]);
    if (tile + kStreamWaves < tile_end) one_tile(tile + kStreamWaves, ld[1]);
  }
}

constexpr int kDeep = 4;  // tiles in flight per wave when a workgroup walks several

// Workgroups of this kernel that fit one XCD (32 compute units) at a time.
static int xcd_slots(int lds_bytes) {
  const int per_cu = (160 * 1024) / lds_bytes;
  return 32 * (per_cu < 2 ? per_cu : 2);   // 2048 threads per compute unit: at most two such workgroups
}

template <int B, bool DUP, bool WIDE_V, bool X_DWORD, int D>
static btc_status launch_lut3(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                              const float* alpha, const float* mu, const void* x, void* y, int y_is_f32, void* ws,
                              int n_ct, int n_rb, int RT, int fin) {
  using Cfg = LutCfg<B, DUP>;
  static_assert(Cfg::kLdsBytes <= 160 * 1024 - 64, "LDS budget");
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemv_lut_kernel<B, DUP, WIDE_V, X_DWORD, D>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  const int grid = ((n_rb + 7) / 8) * 8 * (n_ct + fin);
  gemv_lut_kernel<B, DUP, WIDE_V, X_DWORD, D><<<grid, kWaves * 64, Cfg::kLdsBytes, q>>>(
      d, packed, codebook, alpha, mu, (const __half*)x, y, y_is_f32, carve(ws, d), n_ct, n_rb, RT, fin);
  return launch_status();
}

template <int B, bool DUP, bool WIDE_V, bool X_DWORD>
static btc_status launch_lut2(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                              const float* alpha, const float* mu, const void* x, void* y, int y_is_f32, void* ws) {
  using Cfg = LutCfg<B, DUP>;
  const int n_ct = (d.nchunks + kTileCols - 1) / kTileCols;
  const int tiles = (d.out + kTileRows - 1) / kTileRows;
  // Row blocks (256 rows) per workgroup.  One, as long as all workgroups are resident at once:
  // everything is then requested from memory at the start, which is what a call of a few
  // microseconds needs.  Two beyond that (measured on 7B- to 70B-sized matrices: a second round of
  // workgroups costs more than a second row block, and more than two does not help because a row
  // block costs a workgroup about as much as a table build).  With 10-bit indices the 128 KB
  // table is expensive enough to build once per resident workgroup: then the row blocks are dealt
  // to as many workgroups as stay resident, whole row blocks per XCD.
  const int blocks = (tiles + kRowTiles - 1) / kRowTiles;
  const int slots_xcd = xcd_slots(Cfg::kLdsBytes);
  int RT = 1;
  if (Cfg::kTableBytes >= 128 * 1024) {
    const int rb_xcd = slots_xcd / n_ct;
    const int rb_fit = 8 * (rb_xcd > 0 ? rb_xcd : 1);
    RT = (blocks + rb_fit - 1) / rb_fit;
  } else if ((long long)blocks * n_ct > 8LL * slots_xcd) {
    RT = 2;
  }
  const int n_rb = (blocks + RT - 1) / RT;
  // an extra finishing workgroup per row block, if the grid is still resident at once with it
  const int fin = RT == 1 && (long long)blocks * (n_ct + 1) <= 8LL * slots_xcd;
  if (RT == 1)
    return launch_lut3<B, DUP, WIDE_V, X_DWORD, 1>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws, n_ct, n_rb, RT,
                                                   fin);
  return launch_lut3<B, DUP, WIDE_V, X_DWORD, kDeep>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws, n_ct, n_rb,
                                                     RT, fin);
}

// Streaming variant: applicable when a whole row block's column blocks fit one XCD at one
// workgroup per compute unit, and every wave gets at least two tiles.
template <int B>
static bool stream_applies(const Dims& d, int* n_rb_out, int* tiles_per_wg_out) {
  // Measured on 28672 x 8192: with 9-bit indices (64 KB table, one workgroup per compute unit either
  // way) the streaming kernel takes 21.8 us against 27.0; with 8 bits and fewer the kernel above
  // fits two workgroups per compute unit and wins (17.1 against 20.0 us); the 128 KB table of 10-bit
  // indices leaves no room for 12 staging areas.
  if (B != 9) return false;
  const int n_ct = (d.nchunks + kTileCols - 1) / kTileCols;
  const int tiles = (d.out + kTileRows - 1) / kTileRows;
  if (n_ct + 1 > 32) return false;
  const int n_rb = 8 * (32 / (n_ct + 1));                   // n_ct producers and one finishing workgroup per row block
  const int tiles_per_wg = (tiles + n_rb - 1) / n_rb;
  if (tiles_per_wg < 2 * kStreamWaves) return false;
  *n_rb_out = (tiles + tiles_per_wg - 1) / tiles_per_wg;
  *tiles_per_wg_out = tiles_per_wg;
  return true;
}

template <int B, bool WIDE_V, bool X_DWORD>
static btc_status launch_stream2(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                                 const float* alpha, const float* mu, const void* x, void* y, int y_is_f32, void* ws,
                                 int n_rb, int tiles_per_wg) {
  using Cfg = StreamCfg<B>;
  static_assert(Cfg::kLdsBytes <= 160 * 1024 - 64, "LDS budget");
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemv_lut_stream_kernel<B, WIDE_V, X_DWORD>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  const int n_ct = (d.nchunks + kTileCols - 1) / kTileCols;
  const int grid = ((n_rb + 7) / 8) * 8 * (n_ct + 1);
  gemv_lut_stream_kernel<B, WIDE_V, X_DWORD><<<grid, kStreamWaves * 64, Cfg::kLdsBytes, q>>>(
      d, packed, codebook, alpha, mu, (const __half*)x, y, y_is_f32, carve(ws, d), n_ct, n_rb, tiles_per_wg);
  return launch_status();
}

template <int B>
static btc_status launch_stream(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                                const float* alpha, const float* mu, const void* x, void* y, int y_is_f32, void* ws,
                                int n_rb, int tiles_per_wg) {
  if constexpr (B <= 9) {
    const bool xdw = (d.v % 2 == 0) && (d.in % 2 == 0);
    if (d.v > 16)
      return launch_stream2<B, true, false>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws, n_rb, tiles_per_wg);
    if (xdw)
      return launch_stream2<B, false, true>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws, n_rb, tiles_per_wg);
    return launch_stream2<B, false, false>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws, n_rb, tiles_per_wg);
  } else {
    return BTC_ERR_UNSUPPORTED;
  }
}

template <int B, bool DUP>
static btc_status launch_lut(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                             const float* alpha, const float* mu, const void* x, void* y, int y_is_f32, void* ws) {
  int n_rb, tiles_per_wg;
  if (stream_applies<B>(d, &n_rb, &tiles_per_wg))
    return launch_stream<B>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws, n_rb, tiles_per_wg);
  const bool xdw = (d.v % 2 == 0) && (d.in % 2 == 0);
  if (d.v > 16) return launch_lut2<B, DUP, true, false>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
  if (xdw) return launch_lut2<B, DUP, false, true>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
  return launch_lut2<B, DUP, false, false>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
}

// Index widths with a table that fits LDS, and buffers small enough for 32-bit
// byte offsets with a spare always-out-of-range value.
bool lut_engine_covers(const Dims& d) {
  if (d.b < 5 || d.b > 10) return false;
  if ((long long)d.out * d.wpr * 4 >= (1LL << 31)) return false;
  if ((long long)d.in * 2 >= (1LL << 31) || (long long)d.nchunks * d.v * 2 >= (1LL << 31)) return false;
  const long long n_ct = (d.nchunks + kTileCols - 1) / kTileCols;
  return n_ct * d.out < (1LL << 29);
}

// One activation row; `ws` must hold lut_workspace_bytes() zero bytes (it is left zero).
btc_status gemv_lut(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                    const float* alpha, const float* mu, const void* x, void* y, int y_is_f32, void* ws) {
  switch (d.b) {
    case 5: return launch_lut<5, true>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
    case 6: return launch_lut<6, true>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
    case 7: return launch_lut<7, true>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
    case 8: return launch_lut<8, true>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
    case 9: return launch_lut<9, true>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
    case 10: return launch_lut<10, false>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, ws);
  }
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace btc
