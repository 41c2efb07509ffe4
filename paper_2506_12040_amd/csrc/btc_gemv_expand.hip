// Decode-time product for the tuned settings (chunk length 9 or 10, index
// width 7..10): direct evaluation of the blockwise dot product
//     y_r = sum_j <x_j, C[I_rj]>            (appendix "Binary Codebook LUT-GEMM")
// with the activations held in registers and the codebook expanded to +-1 fp16
// pairs in LDS, so that one chunk costs five packed dot products
// (v_dot2_f32_f16, fp32 accumulate) instead of ten sign-select-and-add steps.
//
// Why not the lookup-and-accumulate scheme of the paper at batch 1: a 7B/13B
// projection streams in a few microseconds.  At that scale a kernel is bound
// by its chain of dependent memory round trips (about a microsecond each) and
// by the serial instruction count of a wave, not by throughput; per-column
// tables need a build phase, a workgroup barrier and a cross-workgroup
// reduction, each of which adds a round trip.  Here a wave owns whole rows,
// needs no workspace and no inter-workgroup traffic, every load of the kernel
// is issued in its first few hundred cycles, and the result is deterministic.
//
// Work split.  Lane l of a wave owns the 32-bit words l, l+64*CS, ... of a
// row's index stream (CS waves of a workgroup may split the columns of long
// rows) and with them the chunks whose b-bit field STARTS in those words.  The
// activations of exactly those chunks sit in registers (zero for chunk slots
// that do not exist, so the row loop has no branch).  The wave then walks over
// its rows: the words of a row are loaded fully coalesced through a buffer
// descriptor, several rows ahead; fields are extracted, each field's five +-1
// pairs are fetched from LDS and accumulated.  Row sums are reduced with DPP;
// the epilogue applies y = alpha * d + mu * sum(x) (dequantisation step of
// Algorithm "Binary Transformation and Compression").
#include <hip/hip_fp16.h>

#include "btc_internal.h"

namespace btc {

typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

namespace expand {

constexpr uint32_t kOob = 0x80000000u;   // buffer offset that is always out of range (buffers are < 2 GiB)
constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format
constexpr int kWaves = 4;                // waves per workgroup
constexpr int kMaxMB = 4;                // words per lane per row, at most
constexpr int kMaxRowsPerGroup = 64;     // rows a wave walks, at most
constexpr int kPD = 4;                   // rows in flight per wave
constexpr int kMaxXBytes = 60 * 1024;    // activations staged in LDS

// Sum over the 64 lanes, valid in lane 63.
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad xor 1
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad xor 2
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false)); // row_bcast:15
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false)); // row_bcast:31
  return v;
}

// B index bits, V chunk length (9 or 10), MB words per lane per row.
template <int B, int V, int MB>
__global__ __launch_bounds__(kWaves * 64) void gemv_expand_kernel(Dims d, const uint32_t* __restrict__ packed,
                                                                 const uint32_t* __restrict__ codebook,
                                                                 const float* __restrict__ alpha,
                                                                 const float* __restrict__ mu,
                                                                 const __half* __restrict__ x, void* __restrict__ y,
                                                                 int y_is_f32, int CS, int rows_per_group, int slot_dwords, int x_vec) {
  constexpr int F = 31 / B + 1;          // fields that can start inside one 32-bit word
  constexpr int VP = (V + 1) / 2;        // fp16 pairs per chunk
  static_assert(VP == 5, "the LDS entry is one 16-byte and one 4-byte read");
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* E = (uint32_t*)smem;                       // codeword k: 5 dwords of +-1 pairs at E[8k]
  uint32_t* xs = E + (1 << B) * 8;                     // activation slots (see below)
  __shared__ float red[kWaves * 2];
  __shared__ float rowpart[kMaxRowsPerGroup * kWaves];

  // every kernel argument is fetched now, in one trip to memory (the empty statement needs them all in registers;
  // left alone the compiler fetches each one next to its first use, one dependent trip after another)
  asm volatile("" ::"s"(packed), "s"(codebook), "s"(alpha), "s"(mu), "s"(x), "s"(y), "s"(y_is_f32), "s"(CS),
               "s"(rows_per_group), "s"(slot_dwords), "s"(x_vec), "s"(d.out), "s"(d.in), "s"(d.wpr), "s"(d.nchunks));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int RG = kWaves / CS;            // row groups (of CS waves) per workgroup
  const int rg = wave / CS, cw = wave - rg * CS;
  const int group = blockIdx.x * RG + rg;
  const int row_begin = group * rows_per_group;

  // ---- per-lane word offsets, then the first rows' index words: issued before anything else
  const uint32_t total_bytes = (uint32_t)d.out * (uint32_t)d.wpr * 4u;
  const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc((void*)packed, 0, (int)total_bytes, kRsrcFlags);
  const uint32_t row_bytes = (uint32_t)d.wpr * 4u;
  uint32_t woff0[MB], woff1[MB], s0[MB];
  int jfirst[MB];
#pragma unroll
  for (int m = 0; m < MB; ++m) {
    const int w = (m * CS + cw) * 64 + lane;               // word index inside a row
    woff0[m] = (w < d.wpr) ? (uint32_t)w * 4u : kOob;
    woff1[m] = (w + 1 < d.wpr) ? (uint32_t)(w + 1) * 4u : kOob;
    jfirst[m] = (32 * w + B - 1) / B;                      // first field that starts in this word
    s0[m] = (uint32_t)(jfirst[m] * B - 32 * w);
  }
  uint32_t w0[kPD][MB], w1[kPD][MB];
  auto load_row = [&](int slot, int row) {                 // rows past the end re-read the last row; never stored
    const uint32_t so = (uint32_t)min(row, d.out - 1) * row_bytes;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
      w0[slot][m] = __builtin_amdgcn_raw_buffer_load_b32(rp, woff0[m], so, 0);
      if (B != 8) w1[slot][m] = __builtin_amdgcn_raw_buffer_load_b32(rp, woff1[m], so, 0);
    }
  };
#pragma unroll
  for (int s = 0; s < kPD; ++s)
    if (s < rows_per_group) load_row(s, row_begin + s);
  // codewords this thread expands, and the scale and mean of the row it will finish: requested
  // now, used after the row loop (a load issued there would add a memory round trip per call)
  constexpr int KPT = ((1 << B) + kWaves * 64 - 1) / (kWaves * 64);
  uint32_t cbv[KPT];
#pragma unroll
  for (int u = 0; u < KPT; ++u) cbv[u] = codebook[min(tid + u * kWaves * 64, (1 << B) - 1)];
  int my_i, my_row;        // the finished row of this thread: row my_i of its group
  if (CS > 1) {
    const int g = tid % RG;
    my_i = tid / RG;
    my_row = my_i < rows_per_group ? (blockIdx.x * RG + g) * rows_per_group + my_i : d.out;
  } else {
    my_i = lane;
    my_row = lane < rows_per_group ? row_begin + lane : d.out;
  }
  const bool my_ok = my_row < d.out;
  const float my_alpha = my_ok ? alpha[my_row] : 0.f;
  const float my_mu = my_ok ? mu[my_row] : 0.f;

  // ---- activations -> LDS, one 5-dword slot per chunk (pairs of fp16; element V of an odd-length
  // chunk is 0), one pad dword after every 4 slots so that lanes reading their slots spread over
  // the banks.  Slot dword i = 5 c + p lives at xs[i + i/20].  Loads past the end of x return 0,
  // so slots nchunks.. are all zero.  Each thread also adds up what it stages.
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, d.in * 2, kRsrcFlags);
  float sx = 0.f;
  const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
  if (V % 2 == 0 && x_vec) {
    // A chunk of 10 fp16 is 5 dwords, so the slot layout is the activation vector itself: copy it
    // 16 bytes at a time (groups of 4 dwords never straddle a pad, which follows every 20th dword).
    const int n4 = (slot_dwords + 3) >> 2;
    const int full4 = (d.in * 2) >> 4;                         // groups that lie entirely inside x
    constexpr int U4 = 3;                                      // 16-byte loads in flight per thread
    for (int base = tid; base < n4; base += kWaves * 64 * U4) {
      uint4 val[U4];
#pragma unroll
      for (int u = 0; u < U4; ++u) {
        const int g = base + u * kWaves * 64;
        if (g < full4) {
          val[u] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rx, (uint32_t)g * 16u, 0, 0));
        } else {                                               // tail group or beyond: dwords past the end read 0
          val[u].x = __builtin_amdgcn_raw_buffer_load_b32(rx, (uint32_t)g * 16u, 0, 0);
          val[u].y = __builtin_amdgcn_raw_buffer_load_b32(rx, (uint32_t)g * 16u + 4u, 0, 0);
          val[u].z = __builtin_amdgcn_raw_buffer_load_b32(rx, (uint32_t)g * 16u + 8u, 0, 0);
          val[u].w = __builtin_amdgcn_raw_buffer_load_b32(rx, (uint32_t)g * 16u + 12u, 0, 0);
        }
      }
#pragma unroll
      for (int u = 0; u < U4; ++u) {
        const int g = base + u * kWaves * 64;
        if (g < n4) {
          uint32_t* dst = xs + 4 * g + g / 5;
          dst[0] = val[u].x; dst[1] = val[u].y; dst[2] = val[u].z; dst[3] = val[u].w;
          sx = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, val[u].x), one, sx, false);
          sx = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, val[u].y), one, sx, false);
          sx = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, val[u].z), one, sx, false);
          sx = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, val[u].w), one, sx, false);
        }
      }
    }
  } else {
    constexpr int U = 8;                                       // loads in flight per thread
    for (int base = tid; base < slot_dwords; base += kWaves * 64 * U) {
      uint32_t val[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = base + u * kWaves * 64;                  // past slot_dwords: reads beyond x, returns 0
        const int c = i / VP, p = i - c * VP;
        const uint32_t e0 = (uint32_t)(c * V + 2 * p) * 2u;
        if (V % 2 == 0) {
          val[u] = __builtin_amdgcn_raw_buffer_load_b32(rx, e0, 0, 0);        // `in` is even: no straddling
        } else {
          const uint32_t lo16 = __builtin_amdgcn_raw_buffer_load_b16(rx, e0, 0, 0);
          const uint32_t hi16 = __builtin_amdgcn_raw_buffer_load_b16(rx, (2 * p + 1 < V) ? e0 + 2u : kOob, 0, 0);
          val[u] = (lo16 & 0xFFFFu) | (hi16 << 16);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = base + u * kWaves * 64;
        if (i < slot_dwords) {
          xs[i + i / 20] = val[u];
          sx = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, val[u]), one, sx, false);
        }
      }
    }
  }
  sx = wave_sum_to_lane63(sx);
  if (lane == 63) red[wave] = sx;
  // ---- codebook -> +-1 fp16 pairs (bit set => +1).  Entries K..2^B-1 are read
  // too: the caller provides 2^B readable entries.
#pragma unroll
  for (int u = 0; u < KPT; ++u) {
    const int k = tid + u * kWaves * 64;
    if (k >= (1 << B)) break;
    const uint32_t npat = ~cbv[u];
    uint32_t e[VP];
#pragma unroll
    for (int p = 0; p < VP; ++p) e[p] = 0x3C003C00u | ((npat >> (2 * p)) & 1u) << 15 | ((npat >> (2 * p + 1)) & 1u) << 31;
    *(uint4*)(E + 8 * k) = make_uint4(e[0], e[1], e[2], e[3]);
    E[8 * k + 4] = e[4];
  }
  __syncthreads();
  sx = 0.f;
#pragma unroll
  for (int wv = 0; wv < kWaves; ++wv) sx += red[wv];         // same order in every wave

  // ---- this lane's activations: chunk slots that do not exist read the all-zero slot `nchunks`
  uint32_t xr[MB][F][VP];
#pragma unroll
  for (int m = 0; m < MB; ++m) {
    const int w = (m * CS + cw) * 64 + lane;
#pragma unroll
    for (int q = 0; q < F; ++q) {
      const int jq = jfirst[m] + q;
      const bool ok = w < d.wpr && jq * B < 32 * (w + 1) && jq < d.nchunks;
      const int c = ok ? jq : d.nchunks;
      const uint32_t* slot = xs + c * VP + (c >> 2);
#pragma unroll
      for (int p = 0; p < VP; ++p) xr[m][q][p] = slot[p];
    }
  }

  // ---- rows; every wave runs the same number of iterations (rows_per_group <= kMaxRowsPerGroup)
  const char* Eb = (const char*)E;
  for (int i0 = 0; i0 < rows_per_group; i0 += kPD) {
#pragma unroll
    for (int s = 0; s < kPD; ++s) {
      const int i = i0 + s;
      if (i >= rows_per_group) break;
      const int row = row_begin + i;
      uint32_t lo[MB], hi[MB];
#pragma unroll
      for (int m = 0; m < MB; ++m) {
        if (B != 8) {
          lo[m] = __builtin_amdgcn_alignbit(w1[s][m], w0[s][m], s0[m]);
          hi[m] = w1[s][m] >> s0[m];
        } else {
          lo[m] = w0[s][m];
          hi[m] = 0;
        }
      }
      if (i + kPD < rows_per_group) load_row(s, row + kPD);  // refill this slot; lo/hi hold the current row
      float acc = 0.f;
#pragma unroll
      for (int m = 0; m < MB; ++m) {
#pragma unroll
        for (int q = 0; q < F; ++q) {
          constexpr uint32_t mask = (1u << B) - 1u;
          const int pos = q * B;
          uint32_t code;
          if (pos + B <= 32) code = (lo[m] >> pos) & mask;
          else code = __builtin_amdgcn_alignbit(hi[m], lo[m], pos) & mask;
          const uint4 e4 = *(const uint4*)(Eb + (code << 5));
          const uint32_t e5 = *(const uint32_t*)(Eb + (code << 5) + 16);
          acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, xr[m][q][0]), __builtin_bit_cast(f16x2, e4.x), acc, false);
          acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, xr[m][q][1]), __builtin_bit_cast(f16x2, e4.y), acc, false);
          acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, xr[m][q][2]), __builtin_bit_cast(f16x2, e4.z), acc, false);
          acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, xr[m][q][3]), __builtin_bit_cast(f16x2, e4.w), acc, false);
          acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, xr[m][q][4]), __builtin_bit_cast(f16x2, e5), acc, false);
        }
      }
      acc = wave_sum_to_lane63(acc);
      if (lane == 63) rowpart[i * kWaves + wave] = acc;      // row sums (or column splits of them) meet in LDS
    }
  }
  // ---- epilogue: thread (row my_i of its group) adds the column splits in a fixed order.  Without a
  // column split the row sums were written by this very wave, so waiting for its own LDS writes is enough.
  if (CS > 1) {
    __syncthreads();
  } else {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if (my_ok) {
    float dsum = 0.f;
    if (CS > 1) {
      const int g = tid % RG;
      for (int c = 0; c < CS; ++c) dsum += rowpart[my_i * kWaves + g * CS + c];
    } else {
      dsum = rowpart[my_i * kWaves + wave];
    }
    const float r = my_alpha * dsum + my_mu * sx;
    if (y_is_f32) ((float*)y)[my_row] = r;
    else ((__half*)y)[my_row] = __float2half_rn(r);
  }
}

// slot dwords staged in LDS: 5 per chunk, plus 4 all-zero slots; and the bytes they take with padding
static int slot_dwords_for(const Dims& d) { return (d.nchunks + 4) * 5; }
static size_t x_lds_bytes_for(const Dims& d) { const int n = slot_dwords_for(d); return (size_t)(n + n / 20 + 4) * 4; }

template <int B, int V, int MB>
static btc_status launch(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                         const float* alpha, const float* mu, const void* x, void* y, int y_is_f32, int CS) {
  const int RG = kWaves / CS;
  // rows per row group: enough groups for ~3 waves per SIMD, at least 2 rows each
  const int target_groups = 256 * 3 * RG;
  int rpg = (d.out + target_groups - 1) / target_groups;
  if (rpg < 2) rpg = 2;
  if (rpg > kMaxRowsPerGroup) rpg = kMaxRowsPerGroup;
  const int groups = (d.out + rpg - 1) / rpg;
  const int grid = (groups + RG - 1) / RG;
  const int xw = slot_dwords_for(d);
  const size_t lds = (size_t)(1 << B) * 32 + x_lds_bytes_for(d);
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemv_expand_kernel<B, V, MB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            32 * 1024 + kMaxXBytes + 256) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  const int x_vec = ((uintptr_t)x & 15) == 0;   // 16-byte loads of the activations
  gemv_expand_kernel<B, V, MB><<<grid, kWaves * 64, lds, q>>>(d, packed, codebook, alpha, mu, (const __half*)x, y,
                                                             y_is_f32, CS, rpg, xw, x_vec);
  return launch_status();
}

template <int B, int V>
static btc_status launch_mb(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                            const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  int CS = 1;
  while (CS < kWaves && (d.wpr + 64 * CS - 1) / (64 * CS) > kMaxMB) CS *= 2;
  const int mb = (d.wpr + 64 * CS - 1) / (64 * CS);
  switch (mb) {
    case 1: return launch<B, V, 1>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, CS);
    case 2: return launch<B, V, 2>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, CS);
    case 3: return launch<B, V, 3>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, CS);
    case 4: return launch<B, V, 4>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32, CS);
  }
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace expand

// Settings with an instantiated kernel, rows short enough for 4 waves x 4 words
// per lane, activations that fit the LDS staging area, and buffers that 32-bit
// byte offsets can address.
bool expand_engine_covers(const Dims& d) {
  if (d.v != 9 && d.v != 10) return false;
  if (d.b < 7 || d.b > 10) return false;
  if (d.wpr > 64 * expand::kWaves * expand::kMaxMB) return false;
  if ((long long)d.out * d.wpr * 4 >= (1LL << 31)) return false;
  if (d.v == 10 && d.in % 2 != 0) return false;   // aligned fp16 pairs
  return expand::x_lds_bytes_for(d) <= (size_t)expand::kMaxXBytes;
}

btc_status gemv_expand(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                       const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  using namespace expand;
#define BTC_EXPAND_CASE(BB, VV) \
  if (d.b == BB && d.v == VV) return launch_mb<BB, VV>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32)
  BTC_EXPAND_CASE(7, 10);
  BTC_EXPAND_CASE(8, 10);
  BTC_EXPAND_CASE(9, 10);
  BTC_EXPAND_CASE(10, 10);
  BTC_EXPAND_CASE(7, 9);
  BTC_EXPAND_CASE(8, 9);
  BTC_EXPAND_CASE(9, 9);
  BTC_EXPAND_CASE(10, 9);
#undef BTC_EXPAND_CASE
  return BTC_ERR_UNSUPPORTED;
}

}  // namespace btc
