// 17..64 activation rows (small-M btc_gemm), chunk length 10, 7..10 index bits: the operand scheme
// of the decode engine (a table entry in LDS IS the A operand of MFMA 16x16x32, chunk-aligned
// permutation of the contraction index: see btc_gemv_mfma.hip), with NB = 2, 3 or 4 blocks of 16
// activation rows as B operands.  An A operand read from the table is used for NB MFMAs.
//
// A workgroup of 16 waves owns 256 weight rows (one block of 16 per wave; two blocks per wave
// on 8 waves measured the same) and a share of the columns, which it walks super-group by super-group (64 chunks) with its accumulators in
// registers: the activations of one super-group (16 NB rows x 640 columns, in operand order) are
// staged in LDS, contracted, and replaced by the next ones, whose global loads were issued a
// whole super-group earlier; the index words of the next super-group are in flight meanwhile.
// Only the column shares (a handful, chosen so that the grid is about one round of compute
// units) leave fp32 partial sums in the workspace for the second pass, which adds them and
// applies alpha and mu (Algorithm "Binary Transformation and Compression": W_hat = alpha * B_hat + mu).
#include "btc_mfma_decode.h"

namespace btc {
namespace rows {

using namespace skinny;   // operand types, table geometry, layout helpers

constexpr int kRWaves = 16;
constexpr int kRR = 1;                  // blocks of 16 weight rows per wave
constexpr int kRowsPerWg = kRWaves * kRR * 16;
constexpr int kV = 10;

template <int B, int NB>
constexpr int rows_lds_bytes() { return Cfg<B>::kE8Bytes + (NB == 2 ? 2 : 1) * NB * kSG * (256 + 64); }

template <int B, int NB, bool BF16>
__global__ __launch_bounds__(kRWaves * 64) void gemm_rows_kernel(
    Dims d, const uint32_t* __restrict__ packed, const uint32_t* __restrict__ codebook,
    const uint16_t* __restrict__ X, int M, int n_cs, int n_rt, int sg_per_cs, int n_rb, float* __restrict__ part,
    float* __restrict__ xpart) {
  using C = Cfg<B>;
  constexpr int NW = C::kNW;
  constexpr int R = kRR;
  constexpr int TPR = 16;                                        // staging tasks (threads) per activation row
  static_assert(kRWaves * 64 >= 16 * NB * TPR, "one staging task per thread at most");
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* E8 = smem;                                      // [code][copy] x 16 B
  // Staged activations of one super-group; with two blocks of activation rows there is room for
  // two such buffers, which lets the next super-group be staged while this one is contracted
  // (one barrier per super-group instead of two).
  constexpr bool DB = NB == 2;
  constexpr int kXBuf = NB * kSG * (256 + 64);                   // bytes of one buffer
  unsigned char* X8 = smem + C::kE8Bytes;                        // [block][chunk][16 rows] x 16 B
  uint32_t* X2 = (uint32_t*)(X8 + NB * kSG * 256);               // [block][chunk / 4][16 rows][chunk % 4] x 4 B: the tails
                                                                 // of the four chunks of a tail MFMA are one 16-byte read

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, q = lane >> 4;
  // Workgroups are dealt round-robin to the 8 XCDs; each XCD gets a contiguous eighth of the
  // (row tile, column share) pairs, so the shares of a row tile mostly meet in one L2, which
  // serves the cache lines that neighbouring shares have in common.
  const int tiles = n_cs * n_rt, xcd = blockIdx.x & 7;
  const int first = (int)((long long)tiles * xcd >> 3), last = (int)((long long)tiles * (xcd + 1) >> 3);
  const int flat = first + (blockIdx.x >> 3);
  if (flat >= last) return;                                      // the grid is padded to 8 x ceil(tiles / 8)
  const int cs = flat % n_cs, rt = flat / n_cs;
  const int sgs = (d.nchunks + kSG - 1) / kSG;
  const int sg_begin = cs * sg_per_cs;
  const int sg_end = min(sgs, sg_begin + sg_per_cs);             // > sg_begin: the host sizes n_cs so
  const int row_base = (rt * kRWaves + wave) * (R * 16);

  // staging role: activation row my_row, pieces my_sub, my_sub + TPR, ...
  const int my_row = tid / TPR, my_sub = tid % TPR;
  const int my_nb = my_row >> 4, my_j = my_row & 15;
  const bool stager = my_row < M && my_row < 16 * NB;
  const __amdgpu_buffer_rsrc_t rX =
      __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, (int)((long long)M * d.in * 2), kRsrcFlags);
  const uint32_t xrow = (uint32_t)my_row * (uint32_t)d.in * 2u;
  // A staging task is four consecutive chunks of one activation row: 80 bytes = five 16-byte
  // loads (rows are only 4-byte aligned, which such loads allow), whose 20 words map to
  // (chunk, slot) at compile time -- no index arithmetic, one 16-byte and one 4-byte LDS
  // write per chunk.  16 tasks per row and super-group; the first 256 NB threads take one each.
  uint4 xv[5];
  auto load_x = [&](int sg) {
    const int k = (sg * kSG + 4 * my_sub) * kV;
#pragma unroll
    for (int m = 0; m < 5; ++m) {
      const uint32_t off = (stager && k + 8 * m < d.in) ? xrow + (uint32_t)(k + 8 * m) * 2u : kOob;
      xv[m] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rX, off, 0, 0));
    }
  };
  float xsum = 0.f;
  auto put_x = [&](int sg) {                                     // operand order; zeros past the end of a row
    const int xb = DB ? ((sg - sg_begin) & 1) * kXBuf : 0;       // byte offset of the buffer of super-group sg
    if (stager) {
      const bool ragged = (sg + 1) * (kSG * kV) > d.in;          // uniform: this super-group reaches past the row's end
      uint32_t w[20] = {xv[0].x, xv[0].y, xv[0].z, xv[0].w, xv[1].x, xv[1].y, xv[1].z, xv[1].w, xv[2].x, xv[2].y,
                        xv[2].z, xv[2].w, xv[3].x, xv[3].y, xv[3].z, xv[3].w, xv[4].x, xv[4].y, xv[4].z, xv[4].w};
      if (ragged) {
        const int k = (sg * kSG + 4 * my_sub) * kV;
#pragma unroll
        for (int u = 0; u < 20; ++u)
          if (k + 2 * u >= d.in) w[u] = 0u;                      // `in` is even here
      }
#pragma unroll
      for (int u = 0; u < 20; ++u) xsum = pair_sum<BF16>(w[u], xsum);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int c = 4 * my_sub + e;
        *(uint4*)(X8 + xb + my_nb * (kSG * 256) + (c * 16 + (my_j ^ (c & 15))) * 16) =
            make_uint4(w[5 * e], w[5 * e + 1], w[5 * e + 2], w[5 * e + 3]);
      }
      // the four tails of the task are the 16 bytes that a tail MFMA reads for this row
      *(uint4*)((unsigned char*)X2 + xb + (my_nb * (kSG * 16) + (my_sub * 16 + my_j) * 4) * 4) = make_uint4(w[4], w[9], w[14], w[19]);
    }
  };
  const __amdgpu_buffer_rsrc_t rP =
      __builtin_amdgcn_make_buffer_rsrc((void*)packed, 0, (int)((uint32_t)d.out * (uint32_t)d.wpr * 4u), kRsrcFlags);
  auto load_w = [&](int sg, uint32_t (&W)[R][NW]) {
    const int cs0 = sg * kSG;
    const int w0 = ((cs0 + 16 * q) * B) >> 5;
    const bool inside = (((cs0 + kSG) * B + 31) >> 5) <= d.wpr;  // uniform: every lane's window lies in its row
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int n = row_base + r * 16 + i;
      const bool row_ok = n < d.out;
      if (inside) {
        const uint32_t off = row_ok ? ((uint32_t)n * (uint32_t)d.wpr + (uint32_t)w0) * 4u : kOob;
        const uint4 v = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rP, off, 0, 0));
        W[r][0] = v.x; W[r][1] = v.y; W[r][2] = v.z; W[r][3] = v.w;
        if constexpr (NW == 5) W[r][4] = __builtin_amdgcn_raw_buffer_load_b32(rP, off + 16u, 0, 0);
      } else {
#pragma unroll
        for (int k = 0; k < NW; ++k) {
          const uint32_t off =
              (row_ok && w0 + k < d.wpr) ? ((uint32_t)n * (uint32_t)d.wpr + (uint32_t)(w0 + k)) * 4u : kOob;
          W[r][k] = __builtin_amdgcn_raw_buffer_load_b32(rP, off, 0, 0);
        }
      }
    }
  };

  // ---- prologue: every load first, then the table, then the first super-group's activations
  constexpr int NC = (C::kK2 + kRWaves * 64 - 1) / (kRWaves * 64);
  uint32_t cw[NC];
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int code = tid + k * kRWaves * 64;
    cw[k] = code < C::kK2 ? codebook[code] : 0u;
  }
  load_x(sg_begin);
  uint32_t Wc[R][NW], Wx[R][NW];
  load_w(sg_begin, Wc);
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int code = tid + k * kRWaves * 64;
    if (code < C::kK2) {
      const uint32_t npat = ~cw[k];
      uint32_t p[4];
#pragma unroll
      for (int m = 0; m < 4; ++m)
        p[m] = (BF16 ? 0x3F803F80u : 0x3C003C00u) | ((npat << (15 - 2 * m)) & 0x8000u) | ((npat << (30 - 2 * m)) & 0x80000000u);
      // the signs of values 8 and 9 ride in the lowest mantissa bit of values 0 and 1
      p[0] |= ((npat >> 8) & 1u) | (((npat >> 9) & 1u) << 16);
#pragma unroll
      for (int c = 0; c < C::kRep; ++c)   // copies in an order rotated by the code: neighbouring threads write different bank groups
        *(uint4*)(E8 + (code * C::kRep + ((c + code) & (C::kRep - 1))) * 16) = make_uint4(p[0], p[1], p[2], p[3]);
    }
  }
  put_x(sg_begin);
  if (sg_begin + 1 < sg_end) load_x(sg_begin + 1);
  __syncthreads();

  // one accumulator per (weight-row block, activation-row block): consecutive MFMAs go to
  // different accumulators, so the chain through one of them never stalls the pipe
  f32x4 acc[R][NB];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[r][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint32_t shift = (uint32_t)(16 * q * B) & 31u;
  typedef __attribute__((address_space(3))) const u32x4* lds_u4;
  const uint32_t e8_lane32 = (uint32_t)(uintptr_t)(lds_u4)(const u32x4*)(E8 + (i & (C::kRep - 1)) * 16);
  const uint32_t x8_lane = (uint32_t)(q * 4096 + i * 16);
  const uint32_t* x2_lane = X2 + (q * 64 + i) * 4;               // tails of chunks 16 q + 4 t .. + 3: + 64 t words
  uint32_t one2;
  if constexpr (BF16) asm volatile("s_mov_b32 %0, 0x3f803f80" : "=s"(one2));
  else asm volatile("s_mov_b32 %0, 0x3c003c00" : "=s"(one2));

  for (int sg = sg_begin; sg < sg_end; ++sg) {
    const bool more = sg + 1 < sg_end;
    const int xb = DB ? ((sg - sg_begin) & 1) * kXBuf : 0;
    if (more) load_w(sg + 1, Wx);
    if (DB && more) {                                            // stage the next super-group into the other buffer
      put_x(sg + 1);
      if (sg + 2 < sg_end) load_x(sg + 2);
    }
    // ---- contraction of super-group sg
    uint32_t Wn[R][NW];
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
      for (int k = 0; k + 1 < NW; ++k) Wn[r][k] = __builtin_amdgcn_alignbit(Wc[r][k + 1], Wc[r][k], shift);
      Wn[r][NW - 1] = Wc[r][NW - 1] >> shift;
    }
    static_for<0, 4>([&](auto t_c) {
      constexpr int t = decltype(t_c)::value;
      uint4 a8[R][4];
      uint32_t a2w[R][4];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        static_for<0, 4>([&](auto w_c) {
          constexpr int w = decltype(w_c)::value;
          constexpr int pos = (4 * t + w) * B;
          constexpr int wi = pos >> 5, sh = pos & 31;
          uint32_t src = Wn[r][wi];
          if constexpr (sh + B > 32) src = __builtin_amdgcn_alignbit(Wn[r][wi + 1 < NW ? wi + 1 : wi], Wn[r][wi], (uint32_t)sh);
          uint32_t code, addr;
          asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(code) : "v"(src), "n"(sh + B > 32 ? 0 : sh), "n"(B));
          asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(addr) : "v"(code), "n"(B <= 8 ? 8 : B == 9 ? 7 : 6), "v"(e8_lane32));
          a8[r][w] = __builtin_bit_cast(uint4, *(lds_u4)(uintptr_t)addr);
        });
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          uint32_t flags;
          asm("v_and_b32 %0, 0x10001, %1" : "=v"(flags) : "v"(a8[r][w].x));
          asm("v_lshl_or_b32 %0, %1, 15, %2" : "=v"(a2w[r][w]) : "v"(flags), "s"(one2));
          a8[r][w].x &= 0xFFFEFFFEu;
        }
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        uint4 b8[4];
        static_for<0, 4>([&](auto w_c) {
          constexpr int w = decltype(w_c)::value;
          constexpr int u = 4 * t + w;
          b8[w] = *(const uint4*)(X8 + xb + nb * (kSG * 256) + ((x8_lane ^ (uint32_t)(u * 16)) + (uint32_t)(u * 256)));
        });
        const uint4 b2 = *(const uint4*)((const unsigned char*)x2_lane + xb + (nb * (kSG * 16) + t * 64) * 4);
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int r = 0; r < R; ++r) acc[r][nb] = mfma16<BF16>(a8[r][w], b8[w], acc[r][nb]);
#pragma unroll
        for (int r = 0; r < R; ++r)
          acc[r][nb] = mfma16<BF16>(make_uint4(a2w[r][0], a2w[r][1], a2w[r][2], a2w[r][3]), b2, acc[r][nb]);
      }
    });
    if (more) {
      __syncthreads();                                           // everybody is done with super-group sg (and, with two
                                                                 // buffers, has staged its part of the next one)
      if (!DB) {
        put_x(sg + 1);
        if (sg + 2 < sg_end) load_x(sg + 2);
        __syncthreads();
      }
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int k = 0; k < NW; ++k) Wc[r][k] = Wx[r][k];
    }
  }

  // ---- partial sums of this column share: lane (j, q) holds weight rows 4 q .. 4 q + 3 of each block
  // for activation row 16 nb + j
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int m = 16 * nb + i;
    if (m < M) {
      float* dst = part + ((size_t)cs * M + m) * d.out;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int n = row_base + r * 16 + 4 * q;
        const f32x4 v = acc[r][nb];
        if ((d.out & 3) == 0) {
          if (n < d.out) *(float4*)(dst + n) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < d.out) dst[n + e] = v[e];
        }
      }
    }
  }
  // ---- sums of the activation rows over this column share (for the mu term): the TPR threads of a
  // row add up; the workgroups of the first row tile leave one copy per block of the second pass
#pragma unroll
  for (int o = TPR / 2; o >= 1; o >>= 1) xsum += __shfl_xor(xsum, o, 64);
  if (rt == 0 && stager)
    for (int nbr = my_sub; nbr < n_rb; nbr += TPR) xpart[((size_t)nbr * n_cs + cs) * 64 + my_row] = xsum;
}

struct RowsPlan {
  int nb;          // blocks of 16 activation rows: 2, 3 or 4
  int n_rt;        // row tiles (256 weight rows)
  int n_cs;        // column shares
  int sg_per_cs;
};

static RowsPlan make_rows_plan(const Dims& d, int M) {
  const int sgs = (d.nchunks + kSG - 1) / kSG;
  RowsPlan p;
  p.nb = M <= 32 ? 2 : M <= 48 ? 3 : 4;
  p.n_rt = (d.out + kRowsPerWg - 1) / kRowsPerWg;
  int n_cs = (256 + p.n_rt - 1) / p.n_rt;                        // about one workgroup per compute unit
  if (n_cs > sgs) n_cs = sgs;
  if (n_cs < 1) n_cs = 1;
  p.sg_per_cs = (sgs + n_cs - 1) / n_cs;
  p.n_cs = (sgs + p.sg_per_cs - 1) / p.sg_per_cs;                // no empty share
  return p;
}

template <int B, int NB, bool BF16>
static btc_status launch_rows(hipStream_t q, const Dims& d, const RowsPlan& pl, const uint32_t* packed,
                              const uint32_t* codebook, const void* X, int M, float* part, float* xpart, int n_rb) {
  static_assert(rows_lds_bytes<B, NB>() <= 160 * 1024 - 64, "LDS budget");
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemm_rows_kernel<B, NB, BF16>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            rows_lds_bytes<B, NB>()) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  gemm_rows_kernel<B, NB, BF16><<<(pl.n_rt * pl.n_cs + 7) / 8 * 8, kRWaves * 64, rows_lds_bytes<B, NB>(), q>>>(
      d, packed, codebook, (const uint16_t*)X, M, pl.n_cs, pl.n_rt, pl.sg_per_cs, n_rb, part, xpart);
  return launch_status();
}

template <int B>
static btc_status launch_rows_b(hipStream_t q, const Dims& d, const RowsPlan& pl, const uint32_t* packed,
                                const uint32_t* codebook, const void* X, int is_bf16, int M, float* part,
                                float* xpart, int n_rb) {
  if (pl.nb == 2) {
    if (is_bf16) return launch_rows<B, 2, true>(q, d, pl, packed, codebook, X, M, part, xpart, n_rb);
    return launch_rows<B, 2, false>(q, d, pl, packed, codebook, X, M, part, xpart, n_rb);
  }
  if (pl.nb == 3) {
    if (is_bf16) return launch_rows<B, 3, true>(q, d, pl, packed, codebook, X, M, part, xpart, n_rb);
    return launch_rows<B, 3, false>(q, d, pl, packed, codebook, X, M, part, xpart, n_rb);
  }
  if (is_bf16) return launch_rows<B, 4, true>(q, d, pl, packed, codebook, X, M, part, xpart, n_rb);
  return launch_rows<B, 4, false>(q, d, pl, packed, codebook, X, M, part, xpart, n_rb);
}

}  // namespace rows

bool gemm_rows_covers(const Dims& d, int M) {
  return M >= 17 && M <= 64 && d.v == rows::kV && d.b >= 7 && d.b <= 10 && (d.in & 1) == 0 &&
         (long long)d.out * d.wpr * 4 < (1LL << 31) && (long long)M * d.in * 2 < (1LL << 31);
}

static size_t rows_xpart_bytes(const Dims& d, const rows::RowsPlan& pl) {
  const int n_rb = (d.out + skinny::kReduceCols - 1) / skinny::kReduceCols;
  return (size_t)n_rb * pl.n_cs * 64 * sizeof(float);
}

size_t gemm_rows_workspace_bytes(const Dims& d, int M) {
  const rows::RowsPlan pl = rows::make_rows_plan(d, M);
  return rows_xpart_bytes(d, pl) + (size_t)pl.n_cs * M * d.out * sizeof(float);
}

// Fitted to measurements on 2.6 .. 26 MB matrices (two launches, prologue, second pass; the index
// stream; what grows with the number of activation rows).
double gemm_rows_estimate_us(const Dims& d, int M) {
  const double bytes = (double)d.out * d.wpr * 4;
  return M <= 32 ? 12.3 + 0.7e-6 * bytes : M <= 48 ? 13.9 + 1.07e-6 * bytes : 15.4 + 1.48e-6 * bytes;
}

btc_status gemm_rows(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook, const float* alpha,
                     const float* mu, const void* X, int is_bf16, int M, void* Y, int y_dtype, void* workspace) {
  using namespace rows;
  const RowsPlan pl = make_rows_plan(d, M);
  const int n_rb = (d.out + skinny::kReduceCols - 1) / skinny::kReduceCols;
  float* xpart = (float*)workspace;
  float* part = (float*)((char*)workspace + rows_xpart_bytes(d, pl));
  btc_status st;
  switch (d.b) {
    case 7: st = launch_rows_b<7>(q, d, pl, packed, codebook, X, is_bf16, M, part, xpart, n_rb); break;
    case 8: st = launch_rows_b<8>(q, d, pl, packed, codebook, X, is_bf16, M, part, xpart, n_rb); break;
    case 9: st = launch_rows_b<9>(q, d, pl, packed, codebook, X, is_bf16, M, part, xpart, n_rb); break;
    case 10: st = launch_rows_b<10>(q, d, pl, packed, codebook, X, is_bf16, M, part, xpart, n_rb); break;
    default: return BTC_ERR_UNSUPPORTED;
  }
  if (st != BTC_OK) return st;
  return skinny_reduce(q, alpha, mu, part, xpart, d.out, M, pl.n_cs, 64, Y, y_dtype);
}

}  // namespace btc
