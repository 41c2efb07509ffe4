// Decode product on the matrix cores: btc_gemv for 2..16 activation rows (and for one row on
// large, very wide matrices), chunk lengths 10 and 9, 7..10 index bits.  (The text describes chunk
// length 10; with 9 the second tail slot of a chunk is a zero in both operands.)
//
// With several activation rows the cost of a call is the decoding of the indices, which does
// not depend on the number of rows, so all rows are served by one pass over the index stream.
// The +-1 patterns go straight from a table in LDS into the A operand of MFMA 16x16x32 (fp16
// in, fp32 accumulate): 16 weight rows x 32 contraction positions per instruction; the
// activation rows (padded to 16) are the B operand.  Nothing is written back to LDS and no lane
// expands a pattern with ALU work: a table entry IS the operand.
//
// The contraction index inside one MFMA may be permuted freely as long as both operands use
// the same permutation.  A chunk has 10 values, an operand register group 8, so the chunks of
// a "super-group" of 64 consecutive chunks are dealt out as follows.  Lane (i, q) -- weight
// row i = lane % 16, group q = lane / 16 -- owns the 16 chunks 16 q .. 16 q + 15 of the
// super-group.  MFMA u (u = 0..15) contracts values 0..7 of chunk 16 q + u in group q; tail
// MFMA t (t = 0..3) contracts values 8 and 9 of the chunks 16 q + 4 t .. + 3.  20 MFMAs cover
// the 640 columns without padding.  Per chunk a lane needs one 16-byte table read: the entry
// holds values 0..7 as +-1.0, and the signs of values 8 and 9 ride in the lowest mantissa bit
// of values 0 and 1, from where two ALU operations turn them into a +-1.0 pair (a third clears
// them, so the entry is exact when it is used).  A lane's 16 indices are one contiguous piece
// of 16 b bits of its row's stream: one 16-byte load (plus one word for b > 8).
//
// Tables: the entries are replicated (16 copies for b <= 8, 8 for b = 9, 4 for b = 10: 64 KB)
// so that the 16 lanes that the LDS serves together read from different bank groups whatever
// their indices are (always for b <= 8, mostly otherwise).
// Activations: staged once per workgroup in operand order, X8[chunk][row] (16 bytes, the row
// position XORed with the chunk number so that both the staging writes and the operand reads
// spread over the banks) and X2[chunk][row] (4 bytes).
//
// Work split: a workgroup (16 waves) owns 256 R weight rows (R blocks of 16 per wave) and up
// to 4 super-groups of columns; the index words of a super-group are requested while the
// previous one is contracted.  The column tiles of a row leave fp32 partial sums in the
// workspace and a second, small kernel adds them, applies alpha and mu (Algorithm "Binary
// Transformation and Compression": W_hat = alpha * B_hat + mu) and clears what it has read.
#include "btc_mfma_decode.h"

namespace btc {
namespace skinny {

template <int V, int B, int R, bool BF16>
__global__ __launch_bounds__(kWaves * 64) void gemv_mfma_kernel(
    Dims d, const uint32_t* __restrict__ packed, const uint32_t* __restrict__ codebook,
    const uint16_t* __restrict__ x, int batch, int n_ct, int n_rt, int nsg, int n_rb, float* __restrict__ part,
    float* __restrict__ xpart) {
  using C = Cfg<B>;
  constexpr int NW = C::kNW;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* E8 = smem;                                      // [code][copy] x 16 B: values 0..7 as +-1 fp16 (+ 2 flag bits)
  unsigned char* X8 = smem + C::kE8Bytes;                        // [chunk][16 rows] x 16 B
  uint32_t* X2 = (uint32_t*)(X8 + nsg * kSG * 256);              // [chunk][16 rows] x 4 B

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, q = lane >> 4;
  // Workgroups are dealt round-robin to the 8 XCDs.  Each XCD gets a contiguous eighth of the
  // tiles in (row tile, column tile) order, so the column tiles of a row tile mostly share an XCD,
  // whose L2 then serves the cache lines that neighbouring tiles have in common: a tile takes
  // only 70..290 bytes of a row (measured without this: 2.0x the index stream fetched).
  const int tiles = n_ct * n_rt, xcd = blockIdx.x & 7;
  const int first = (int)((long long)tiles * xcd >> 3), last = (int)((long long)tiles * (xcd + 1) >> 3);
  const int flat = first + (blockIdx.x >> 3);
  if (flat >= last) return;                                      // the grid is padded to 8 x ceil(tiles / 8)
  const int ct = flat % n_ct, rt = flat / n_ct;
  const int sgs = (d.nchunks + kSG - 1) / kSG;
  const int my_nsg = min(nsg, sgs - ct * nsg);                   // >= 1: the host sizes n_ct so
  const int c0 = ct * nsg * kSG;                                 // first chunk of this column tile
  const int row_base = (rt * kWaves + wave) * (R * 16);

  // ---- every global load of the prologue is issued before anything waits: codebook, this
  // tile's activations, then the index words super-group by super-group.  Loads return in
  // order, so the tables can be built and the activations staged while the index words are
  // still arriving, and the contraction of a super-group starts as soon as its words are
  // there while the later ones stream in.
  constexpr int NC = (C::kK2 + kWaves * 64 - 1) / (kWaves * 64);
  uint32_t cw[NC];
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int code = tid + k * kWaves * 64;
    cw[k] = code < C::kK2 ? codebook[code] : 0u;
  }
  // activations: wave w stages row w, a lane takes 16-byte pieces of it
  static_assert(V == 9 || V == 10, "chunk lengths 9 (one tail value) and 10 (two)");
  constexpr int NS = (kMaxSG * (kSG * V / 8) + 63) / 64;         // pieces per lane and row
  const int nseg = my_nsg * (kSG * V / 8);
  const int k0 = c0 * V;
  uint4 xv[NS];
  {
    const __amdgpu_buffer_rsrc_t rX =
        __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)((long long)batch * d.in * 2), kRsrcFlags);
    const uint32_t rowoff = (uint32_t)wave * (uint32_t)d.in * 2u;
#pragma unroll
    for (int m = 0; m < NS; ++m) {
      const int seg = lane + 64 * m;
      const int k = k0 + 8 * seg;
      const uint32_t off = (wave < batch && seg < nseg && k < d.in) ? rowoff + (uint32_t)k * 2u : kOob;
      xv[m] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rX, off, 0, 0));
    }
  }
  const __amdgpu_buffer_rsrc_t rP =
      __builtin_amdgcn_make_buffer_rsrc((void*)packed, 0, (int)((uint32_t)d.out * (uint32_t)d.wpr * 4u), kRsrcFlags);
  uint32_t W[kMaxSG][R][NW];
  auto load_words = [&](auto sg_c) {
    constexpr int sg = decltype(sg_c)::value;
    const int cs = c0 + sg * kSG;
    const int w0 = ((cs + 16 * q) * B) >> 5;
    // does every lane's window of NW words lie inside its row?  (uniform; false only in the last
    // super-group of a row, where words are fetched one by one and those past the row read as zero)
    const bool inside = (((cs + kSG) * B + 31) >> 5) <= d.wpr;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int n = row_base + r * 16 + i;
      const bool row_ok = sg < my_nsg && n < d.out;
      if (inside) {
        const uint32_t off = row_ok ? ((uint32_t)n * (uint32_t)d.wpr + (uint32_t)w0) * 4u : kOob;
        const uint4 v = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rP, off, 0, 0));
        W[sg][r][0] = v.x; W[sg][r][1] = v.y; W[sg][r][2] = v.z; W[sg][r][3] = v.w;
        if constexpr (NW == 5) W[sg][r][4] = __builtin_amdgcn_raw_buffer_load_b32(rP, off + 16u, 0, 0);
      } else {
#pragma unroll
        for (int k = 0; k < NW; ++k) {
          const uint32_t off =
              (row_ok && w0 + k < d.wpr) ? ((uint32_t)n * (uint32_t)d.wpr + (uint32_t)(w0 + k)) * 4u : kOob;
          W[sg][r][k] = __builtin_amdgcn_raw_buffer_load_b32(rP, off, 0, 0);
        }
      }
    }
  };

  // ---- pattern tables: a thread writes all copies of its entries
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int code = tid + k * kWaves * 64;
    if (code < C::kK2) {
      const uint32_t npat = ~cw[k];
      uint32_t p[4];
#pragma unroll
      for (int m = 0; m < 4; ++m)
        p[m] = (BF16 ? 0x3F803F80u : 0x3C003C00u) | ((npat << (15 - 2 * m)) & 0x8000u) | ((npat << (30 - 2 * m)) & 0x80000000u);
      // the signs of values 8 and 9 ride in the lowest mantissa bit of values 0 and 1; the reader
      // moves them into a +-1 pair of its own and clears them before the entry is used
      p[0] |= ((npat >> 8) & 1u) | (V == 10 ? ((npat >> 9) & 1u) << 16 : 0u);
#pragma unroll
      for (int c = 0; c < C::kRep; ++c)   // copies in an order rotated by the code: neighbouring threads write different bank groups
        *(uint4*)(E8 + (code * C::kRep + ((c + code) & (C::kRep - 1))) * 16) = make_uint4(p[0], p[1], p[2], p[3]);
    }
  }

  // ---- activations into operand order.  Columns past the end of a row are staged as zeros,
  // which is what makes the padding of the last chunk and the chunks past the end of the row
  // contribute nothing.  Chunk length 10: pair by pair (a pair never straddles a chunk; rows have
  // an even number of columns here).  Chunk length 9: value by value; the second tail slot is zero
  // (and so is the table's).
  if (wave < batch) {
    const int j = wave;
    if constexpr (V == 10) {
      auto put = [&](int p, uint32_t w) {                        // pair p of the tile: values 2p, 2p+1
        const int c = (int)(((uint32_t)p * 52429u) >> 18);       // p / 5 for p < 2^16
        const int s = p - 5 * c;
        if (k0 + 2 * p >= d.in) w = 0u;
        if (s < 4) ((uint32_t*)X8)[(c * 16 + (j ^ (c & 15))) * 4 + s] = w;
        else X2[x2_word(c, j)] = w;
      };
#pragma unroll
      for (int m = 0; m < NS; ++m) {
        const int seg = lane + 64 * m;
        if (seg < nseg) {
          put(4 * seg + 0, xv[m].x); put(4 * seg + 1, xv[m].y);
          put(4 * seg + 2, xv[m].z); put(4 * seg + 3, xv[m].w);
        }
      }
    } else {
      auto put = [&](int e, uint32_t h) {                        // value e of the tile (16 bits)
        const int c = e / V, t = e - V * c;
        if (k0 + e >= d.in) h = 0u;
        if (t < 8) ((uint16_t*)X8)[(c * 16 + (j ^ (c & 15))) * 8 + t] = (uint16_t)h;
        else X2[x2_word(c, j)] = h;
      };
#pragma unroll
      for (int m = 0; m < NS; ++m) {
        const int seg = lane + 64 * m;
        if (seg < nseg) {
          const uint32_t w[4] = {xv[m].x, xv[m].y, xv[m].z, xv[m].w};
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            put(8 * seg + 2 * u, w[u] & 0xFFFFu);
            put(8 * seg + 2 * u + 1, w[u] >> 16);
          }
        }
      }
    }
  }
  static_for<0, kAhead>([&](auto sg_c) { load_words(sg_c); });
  __syncthreads();

  // ---- sums of the activation rows over this column tile (for the mu term), once per tile:
  // the workgroups of the first row tile leave one copy per block of the second pass
  if (rt == 0 && wave < batch) {
    const int j = wave;
    float s = 0.f;
    for (int c = lane; c < my_nsg * kSG; c += 64) {
      const uint4 v = *(const uint4*)(X8 + (c * 16 + (j ^ (c & 15))) * 16);
      s = pair_sum<BF16>(v.x, s); s = pair_sum<BF16>(v.y, s); s = pair_sum<BF16>(v.z, s); s = pair_sum<BF16>(v.w, s);
      s = pair_sum<BF16>(X2[x2_word(c, j)], s);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
    for (int nb = lane; nb < n_rb; nb += 64) xpart[((size_t)nb * n_ct + ct) * 16 + j] = s;
  }

  // ---- contraction
  f32x4 acc[R][2];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    acc[r][0] = f32x4{0.f, 0.f, 0.f, 0.f};
    acc[r][1] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const uint32_t shift = (uint32_t)(16 * q * B) & 31u;           // where the lane's first index starts in its window
  typedef __attribute__((address_space(3))) const u32x4* lds_u4;
  const uint32_t e8_lane32 = (uint32_t)(uintptr_t)(lds_u4)(const u32x4*)(E8 + (i & (C::kRep - 1)) * 16);   // LDS address of the lane's copy of entry 0
  // Lane-dependent parts of the operand addresses, so that the loops add constants only: chunk
  // cl = 64 sg + 16 q + u sits at X8 + 256 cl + 16 (i ^ u) and at word x2_word(cl, i) of X2.
  const uint32_t x8_lane = (uint32_t)(q * 4096 + i * 16);
  const uint32_t* x2_lane[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) x2_lane[w] = X2 + q * 256 + ((w + q) & 3) * 16 + i;
  uint32_t one2;                                                 // 1.0 | 1.0 in a scalar register: an instruction takes one literal only
  // (chunk length 9: the second tail slot is 0.0)
  if constexpr (BF16) {
    if constexpr (V == 10) asm volatile("s_mov_b32 %0, 0x3f803f80" : "=s"(one2));
    else asm volatile("s_mov_b32 %0, 0x00003f80" : "=s"(one2));
  } else {
    if constexpr (V == 10) asm volatile("s_mov_b32 %0, 0x3c003c00" : "=s"(one2));
    else asm volatile("s_mov_b32 %0, 0x00003c00" : "=s"(one2));
  }
  static_for<0, kMaxSG>([&](auto sg_c) {
    constexpr int sg = decltype(sg_c)::value;
    if constexpr (sg + kAhead < kMaxSG) {
      if (sg + kAhead < my_nsg) load_words(std::integral_constant<int, sg + kAhead>{});
    }
    if (sg < my_nsg) {
      // the lane's 16 indices, aligned to bit 0 of Wn
      uint32_t Wn[R][NW];
#pragma unroll
      for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int k = 0; k + 1 < NW; ++k) Wn[r][k] = __builtin_amdgcn_alignbit(W[sg][r][k + 1], W[sg][r][k], shift);
        Wn[r][NW - 1] = W[sg][r][NW - 1] >> shift;
      }
      static_for<0, 4>([&](auto t_c) {
        constexpr int t = decltype(t_c)::value;
        uint4 b8[4], b2;
        uint32_t b2w[4];
        static_for<0, 4>([&](auto w_c) {
          constexpr int w = decltype(w_c)::value;
          constexpr int u = 4 * t + w;
          b8[w] = *(const uint4*)(X8 + ((x8_lane ^ (uint32_t)(u * 16)) + (uint32_t)((sg * kSG + u) * 256)));
          b2w[w] = x2_lane[w][(16 * sg + t) * 64];
        });
        b2 = make_uint4(b2w[0], b2w[1], b2w[2], b2w[3]);
        // all table reads of this step first (R x 4 independent reads in flight), then the
        // fix-ups, then the matrix instructions
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
            // code = bits [sh, sh + B) of src; entry address = lane base + code * (copies * 16)
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
        for (int r = 0; r < R; ++r) {
          acc[r][0] = mfma16<BF16>(a8[r][0], b8[0], acc[r][0]);
          acc[r][1] = mfma16<BF16>(a8[r][1], b8[1], acc[r][1]);
          acc[r][0] = mfma16<BF16>(a8[r][2], b8[2], acc[r][0]);
          acc[r][1] = mfma16<BF16>(a8[r][3], b8[3], acc[r][1]);
          acc[r][0] = mfma16<BF16>(make_uint4(a2w[r][0], a2w[r][1], a2w[r][2], a2w[r][3]), b2, acc[r][0]);
        }
      });
    }
  });

  // ---- partial sums: lane (j, q) holds the weight rows 4 q .. 4 q + 3 of each block for activation row j
  if (i < batch) {
    float* dst = part + ((size_t)ct * batch + i) * d.out;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int n = row_base + r * 16 + 4 * q;
      const f32x4 v = acc[r][0] + acc[r][1];
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

// Second pass: y[j][n] = alpha[n] * (sum of the column tiles' partial sums) + mu[n] * (sum of row j).
// A block owns kReduceCols outputs of one activation row and its own copies of the row sums, so
// it can clear what it has read without a race.  Its four waves share the column tiles (wave g
// takes tiles g, g + 4, ...), each lane four consecutive outputs; wave 0 adds the four results.
// (A finishing workgroup inside the first kernel instead of this pass was tried: partial sums
// that cross XCDs inside one kernel need agent-scope accesses or cache write-backs, and both
// cost more than the second launch.)
__global__ __launch_bounds__(256) void skinny_reduce_kernel(const float* __restrict__ alpha, const float* __restrict__ mu,
                                                            float* __restrict__ part, float* __restrict__ xpart, int out,
                                                            int batch, int n_ct, int xstride, void* __restrict__ y, int y_dtype) {
  __shared__ float4 red[3][64];
  const int nb = blockIdx.x, j = blockIdx.y, tid = threadIdx.x, lane = tid & 63, g = tid >> 6;
  const int n_end = min(out, (nb + 1) * kReduceCols);
  const size_t yrow = (size_t)j * out;
  float xs = 0.f;
  if (g == 0) {                                      // the row sum: one tile per lane, then across the wave
    for (int ct = lane; ct < n_ct; ct += 64) xs += xpart[((size_t)nb * n_ct + ct) * xstride + j];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) xs += __shfl_xor(xs, o, 64);
  }
  if ((out & 3) == 0) {
    const int n = nb * kReduceCols + 4 * lane;
    const bool ok = n < n_end;
    float4 al = make_float4(0.f, 0.f, 0.f, 0.f), mn = al, v = al;
    if (ok && g == 0) {
      al = *(const float4*)(alpha + n);
      mn = *(const float4*)(mu + n);
    }
    if (ok) {
      float4* p0 = (float4*)(part + (size_t)j * out + n);
      const size_t step = (size_t)batch * out / 4;   // float4s between consecutive column tiles
      for (int ct = g; ct < n_ct; ct += 16) {        // four tiles of this wave at a time: loads first, then clears
        float4 t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          t[u] = ct + 4 * u < n_ct ? p0[(size_t)(ct + 4 * u) * step] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          v.x += t[u].x; v.y += t[u].y; v.z += t[u].z; v.w += t[u].w;
          if (ct + 4 * u < n_ct) p0[(size_t)(ct + 4 * u) * step] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
    }
    if (g > 0) red[g - 1][lane] = v;
    __syncthreads();
    if (g == 0 && ok) {
#pragma unroll
      for (int u = 0; u < 3; ++u) {
        const float4 t = red[u][lane];
        v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
      }
      const float r0 = al.x * v.x + mn.x * xs, r1 = al.y * v.y + mn.y * xs, r2 = al.z * v.z + mn.z * xs,
                  r3 = al.w * v.w + mn.w * xs;
      if (y_dtype == BTC_F32) {
        *(float4*)((float*)y + yrow + n) = make_float4(r0, r1, r2, r3);
      } else if (y_dtype == BTC_BF16) {
        *(uint2*)((uint16_t*)y + yrow + n) =
            make_uint2(bf16_bits(r0) | (bf16_bits(r1) << 16), bf16_bits(r2) | (bf16_bits(r3) << 16));
      } else {
        const __half2 h0 = __floats2half2_rn(r0, r1), h1 = __floats2half2_rn(r2, r3);
        *(uint2*)((uint16_t*)y + yrow + n) =
            make_uint2(__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1));
      }
    }
  } else {
    if (g == 0) {
      for (int n = nb * kReduceCols + lane; n < n_end; n += 64) {
        float v = 0.f;
        for (int ct = 0; ct < n_ct; ++ct) {
          float* p = part + ((size_t)ct * batch + j) * out + n;
          v += *p;
          *p = 0.f;
        }
        const float r = alpha[n] * v + mu[n] * xs;
        if (y_dtype == BTC_F32) ((float*)y)[yrow + n] = r;
        else if (y_dtype == BTC_BF16) ((__hip_bfloat16*)y)[yrow + n] = __float2bfloat16(r);
        else ((__half*)y)[yrow + n] = __float2half_rn(r);
      }
    }
  }
  // the row sums are read by wave 0 only, which clears them afterwards
  if (g == 0)
    for (int ct = lane; ct < n_ct; ct += 64) xpart[((size_t)nb * n_ct + ct) * xstride + j] = 0.f;
}

// ---------------------------------------------------------------------------------------------
// One activation row, one kernel: the same operand scheme with a workgroup of 8 waves that owns
// 16 weight rows over ALL columns.  Wave w takes the super-groups w, w + 8, ... (the sums of the
// eight waves meet in LDS), so no partial sum leaves the workgroup and the call is a single
// launch whose chain is: every load issued at once, one wait, table and staging, a handful of
// MFMAs per wave, 16 outputs.  The activation row (20 bytes per chunk) and a 32 KB table fit
// two to three workgroups per compute unit.  All 16 columns of the B operand read the same
// activation row (one LDS address per lane group: a broadcast), so every column of the result
// is the answer and column 0 is taken.
constexpr int kOneWaves = 8;
constexpr int kOneIters = 8;            // super-groups per wave at most: in <= 8 * 8 * 640 columns (chunk length 10)
constexpr int kOnePieces = 8;           // 16-byte pieces of the activation row per thread at most

template <int B>
struct OneCfg {
  static constexpr int kRep = (2048 >> B) > 16 ? 16 : (2048 >> B);        // copies of a 16-byte entry: 32 KB
  static constexpr int kE8Bytes = (1 << B) * kRep * 16;
};

constexpr int one_lds_bytes(int e8, int sgs) { return e8 + sgs * kSG * 20 + kOneWaves * 16 * 4 * 4 + 64; }

template <int V, int B, int R>
__global__ __launch_bounds__(kOneWaves * 64) void gemv_mfma_one_kernel(
    Dims d, const uint32_t* __restrict__ packed, const uint32_t* __restrict__ codebook,
    const float* __restrict__ alpha, const float* __restrict__ mu, const uint16_t* __restrict__ x,
    void* __restrict__ y, int y_is_f32) {
  static_assert(V == 9 || V == 10, "chunk lengths 9 and 10");
  using C = OneCfg<B>;
  constexpr int NW = Cfg<B>::kNW;
  constexpr int K2 = 1 << B;
  extern __shared__ __align__(16) unsigned char smem[];
  const int sgs = (d.nchunks + kSG - 1) / kSG;
  unsigned char* E8 = smem;                                      // [code][copy] x 16 B
  unsigned char* X8 = smem + C::kE8Bytes;                        // [chunk] x 16 B: values 0..7
  uint32_t* X2 = (uint32_t*)(X8 + sgs * kSG * 16);               // [chunk] x 4 B: values 8, 9
  float* red = (float*)(X2 + sgs * kSG);                         // [wave][16 R rows]
  float* xs_w = red + kOneWaves * 16 * R;                            // [wave]: partial sums of the activation row

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, q = lane >> 4;
  const int n0 = blockIdx.x * (16 * R);                          // first weight row of the workgroup

  // ---- every global load first
  constexpr int NC = (K2 + kOneWaves * 64 - 1) / (kOneWaves * 64);
  uint32_t cw[NC];
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int code = tid + k * kOneWaves * 64;
    cw[k] = code < K2 ? codebook[code] : 0u;
  }
  const __amdgpu_buffer_rsrc_t rX = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, d.in * 2, kRsrcFlags);
  uint4 xv[kOnePieces];
#pragma unroll
  for (int m = 0; m < kOnePieces; ++m) {
    const int k = 8 * (tid + m * kOneWaves * 64);
    xv[m] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rX, k < d.in ? (uint32_t)k * 2u : kOob, 0, 0));
  }
  const __amdgpu_buffer_rsrc_t rP =
      __builtin_amdgcn_make_buffer_rsrc((void*)packed, 0, (int)((uint32_t)d.out * (uint32_t)d.wpr * 4u), kRsrcFlags);
  uint32_t W[kOneIters][R][NW];
#pragma unroll
  for (int it = 0; it < kOneIters; ++it) {
    const int sg = wave + it * kOneWaves;
    const int cs = sg * kSG;
    const int w0 = ((cs + 16 * q) * B) >> 5;
    const bool inside = (((cs + kSG) * B + 31) >> 5) <= d.wpr;   // uniform: the whole window of every lane lies in its row
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int n = n0 + 16 * r + i;
      const bool row_ok = sg < sgs && n < d.out;
      if (inside) {
        const uint32_t off = row_ok ? ((uint32_t)n * (uint32_t)d.wpr + (uint32_t)w0) * 4u : kOob;
        const uint4 v = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rP, off, 0, 0));
        W[it][r][0] = v.x; W[it][r][1] = v.y; W[it][r][2] = v.z; W[it][r][3] = v.w;
        if constexpr (NW == 5) W[it][r][4] = __builtin_amdgcn_raw_buffer_load_b32(rP, off + 16u, 0, 0);
      } else {
#pragma unroll
        for (int k = 0; k < NW; ++k) {
          const uint32_t off =
              (row_ok && w0 + k < d.wpr) ? ((uint32_t)n * (uint32_t)d.wpr + (uint32_t)(w0 + k)) * 4u : kOob;
          W[it][r][k] = __builtin_amdgcn_raw_buffer_load_b32(rP, off, 0, 0);
        }
      }
    }
  }
  const float my_alpha = (tid < 16 * R && n0 + tid < d.out) ? alpha[n0 + tid] : 0.f;
  const float my_mu = (tid < 16 * R && n0 + tid < d.out) ? mu[n0 + tid] : 0.f;

  // ---- table
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int code = tid + k * kOneWaves * 64;
    if (code < K2) {
      const uint32_t npat = ~cw[k];
      uint32_t p[4];
#pragma unroll
      for (int m = 0; m < 4; ++m)
        p[m] = 0x3C003C00u | ((npat << (15 - 2 * m)) & 0x8000u) | ((npat << (30 - 2 * m)) & 0x80000000u);
      p[0] |= ((npat >> 8) & 1u) | (V == 10 ? ((npat >> 9) & 1u) << 16 : 0u);
#pragma unroll
      for (int c = 0; c < C::kRep; ++c)   // copies in an order rotated by the code: neighbouring threads write different bank groups
        *(uint4*)(E8 + (code * C::kRep + ((c + code) & (C::kRep - 1))) * 16) = make_uint4(p[0], p[1], p[2], p[3]);
    }
  }
  // ---- the activation row into operand order (zeros past its end), and its sum
  float xsum = 0.f;
  {
    const int n_vals = sgs * kSG * V;                            // slots of the staged row
#pragma unroll
    for (int m = 0; m < kOnePieces; ++m) {
      const int k = 8 * (tid + m * kOneWaves * 64);
      if (k < n_vals) {
        const uint32_t w[4] = {xv[m].x, xv[m].y, xv[m].z, xv[m].w};
        if constexpr (V == 10) {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int p = k / 2 + u;                             // pair p: values 2p, 2p+1 (never straddles a chunk)
            const uint32_t wv = 2 * p < d.in ? w[u] : 0u;        // `in` is even here
            xsum = pair_sum<false>(wv, xsum);
            const int c = (int)(((uint32_t)p * 52429u) >> 18), sl = p - 5 * c;
            if (sl < 4) ((uint32_t*)X8)[c * 4 + sl] = wv;
            else X2[c] = wv;
          }
        } else {
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int e = k + u;
            uint32_t h = (u & 1) ? w[u >> 1] >> 16 : w[u >> 1] & 0xFFFFu;
            if (e >= d.in) h = 0u;
            xsum = pair_sum<false>(h, xsum);
            const int c = e / V, t = e - V * c;
            if (t < 8) ((uint16_t*)X8)[c * 8 + t] = (uint16_t)h;
            else X2[c] = h;
          }
        }
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) xsum += __shfl_xor(xsum, o, 64);
    if (lane == 0) xs_w[wave] = xsum;
  }
  __syncthreads();

  // ---- contraction: this wave's super-groups
  f32x4 acc[R][2];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r][0] = acc[r][1] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint32_t shift = (uint32_t)(16 * q * B) & 31u;
  typedef __attribute__((address_space(3))) const u32x4* lds_u4;
  const uint32_t e8_lane32 = (uint32_t)(uintptr_t)(lds_u4)(const u32x4*)(E8 + (i & (C::kRep - 1)) * 16);
  uint32_t one2;
  if constexpr (V == 10) asm volatile("s_mov_b32 %0, 0x3c003c00" : "=s"(one2));
  else asm volatile("s_mov_b32 %0, 0x00003c00" : "=s"(one2));
  static_for<0, kOneIters>([&](auto it_c) {
    constexpr int it = decltype(it_c)::value;
    const int sg = wave + it * kOneWaves;
    if (sg < sgs) {
      uint32_t Wn[R][NW];
#pragma unroll
      for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int k = 0; k + 1 < NW; ++k) Wn[r][k] = __builtin_amdgcn_alignbit(W[it][r][k + 1], W[it][r][k], shift);
        Wn[r][NW - 1] = W[it][r][NW - 1] >> shift;
      }
      const unsigned char* xb8 = X8 + (sg * kSG + 16 * q) * 16;  // the lane group's 16 chunks (the same for all 16 columns)
      const uint32_t* xb2 = X2 + sg * kSG + 16 * q;
      static_for<0, 4>([&](auto t_c) {
        constexpr int t = decltype(t_c)::value;
        uint4 a8[R][4], b8[4];
        uint32_t a2w[R][4];
#pragma unroll
        for (int w = 0; w < 4; ++w) b8[w] = *(const uint4*)(xb8 + (4 * t + w) * 16);
        const uint4 b2 = *(const uint4*)(xb2 + 4 * t);
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
            asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(addr) : "v"(code), "n"(B <= 7 ? 8 : B == 8 ? 7 : B == 9 ? 6 : 5), "v"(e8_lane32));
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
        for (int r = 0; r < R; ++r) {
          acc[r][0] = mfma16<false>(a8[r][0], b8[0], acc[r][0]);
          acc[r][1] = mfma16<false>(a8[r][1], b8[1], acc[r][1]);
          acc[r][0] = mfma16<false>(a8[r][2], b8[2], acc[r][0]);
          acc[r][1] = mfma16<false>(a8[r][3], b8[3], acc[r][1]);
          acc[r][0] = mfma16<false>(make_uint4(a2w[r][0], a2w[r][1], a2w[r][2], a2w[r][3]), b2, acc[r][0]);
        }
      });
    }
  });

  // ---- the eight waves' sums meet in LDS; 16 threads finish the 16 rows
  if (i == 0) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const f32x4 v = acc[r][0] + acc[r][1];                     // column 0: weight rows 4 q .. 4 q + 3 of block r
      *(float4*)(red + (wave * R + r) * 16 + 4 * q) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
  __syncthreads();
  if (tid < 16 * R) {
    float sum = 0.f, sx = 0.f;
#pragma unroll
    for (int w = 0; w < kOneWaves; ++w) {
      sum += red[w * 16 * R + tid];
      sx += xs_w[w];
    }
    const int nn = n0 + tid;
    if (nn < d.out) {
      const float r = my_alpha * sum + my_mu * sx;
      if (y_is_f32) ((float*)y)[nn] = r;
      else ((__half*)y)[nn] = __float2half_rn(r);
    }
  }
}

struct Plan {
  int R;        // blocks of 16 weight rows per wave
  int nsg;      // super-groups per column tile
  int n_ct;     // column tiles
  int n_rt;     // row tiles
  double est_us;
};

// Tile shape: the kernel lasts about rounds x (fixed + R nsg unit), one workgroup per compute unit;
// fixed = tables and staging, unit = one block of 16 rows x 64 chunks on each of the 8 waves.
static Plan make_plan(const Dims& d) {
  const int sgs = (d.nchunks + kSG - 1) / kSG;
  Plan best{0, 0, 0, 0, 1e30};
  for (int R = 1; R <= 2; R *= 2)
    for (int nsg = 1; nsg <= kMaxSG; ++nsg) {
      const int n_ct = (sgs + nsg - 1) / nsg;
      const int n_rt = (d.out + kWaves * R * 16 - 1) / (kWaves * R * 16);
      const double rounds = (double)(((long long)n_ct * n_rt + 255) / 256);
      const double t = rounds * (2.0 + 0.9 * R * nsg) + 0.15 * n_ct;   // + the second pass reading n_ct partial sums
      if (t < best.est_us) best = Plan{R, nsg, n_ct, n_rt, t};
    }
  return best;
}

template <int V, int B, int R, bool BF16>
static btc_status launch2(hipStream_t q, const Dims& d, const Plan& pl, const uint32_t* packed, const uint32_t* codebook,
                          const void* x, int batch, float* part, float* xpart, int n_rb) {
  using C = Cfg<B>;
  static_assert(lds_bytes(C::kE8Bytes, kMaxSG) <= 160 * 1024 - 64, "LDS budget");
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemv_mfma_kernel<V, B, R, BF16>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            lds_bytes(C::kE8Bytes, kMaxSG)) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  gemv_mfma_kernel<V, B, R, BF16><<<(pl.n_ct * pl.n_rt + 7) / 8 * 8, kWaves * 64, lds_bytes(C::kE8Bytes, pl.nsg), q>>>(
      d, packed, codebook, (const uint16_t*)x, batch, pl.n_ct, pl.n_rt, pl.nsg, n_rb, part, xpart);
  return launch_status();
}

template <int V, int B>
static btc_status launch1(hipStream_t q, const Dims& d, const Plan& pl, const uint32_t* packed, const uint32_t* codebook,
                          const void* x, int is_bf16, int batch, float* part, float* xpart, int n_rb) {
  if (is_bf16) {
    if (pl.R == 1) return launch2<V, B, 1, true>(q, d, pl, packed, codebook, x, batch, part, xpart, n_rb);
    return launch2<V, B, 2, true>(q, d, pl, packed, codebook, x, batch, part, xpart, n_rb);
  }
  if (pl.R == 1) return launch2<V, B, 1, false>(q, d, pl, packed, codebook, x, batch, part, xpart, n_rb);
  return launch2<V, B, 2, false>(q, d, pl, packed, codebook, x, batch, part, xpart, n_rb);
}

}  // namespace skinny

// Single-row, single-kernel variant: the staged row and the table must fit LDS with room for a
// second workgroup, a wave takes at most kOneIters super-groups, and the threads' 16-byte pieces
// must cover every staged slot.
bool gemv_mfma_one_covers(const Dims& d) {
  const int sgs = (d.nchunks + skinny::kSG - 1) / skinny::kSG;
  return (d.v == 9 || d.v == 10) && d.b >= 7 && d.b <= 10 && (d.in & 1) == 0 &&
         sgs <= skinny::kOneWaves * skinny::kOneIters &&
         sgs * skinny::kSG * d.v <= 8 * skinny::kOnePieces * skinny::kOneWaves * 64 &&
         skinny::one_lds_bytes(32 << 10, sgs) <= 80 * 1024 && (long long)d.out * d.wpr * 4 < (1LL << 31);
}

template <int V, int B, int R>
static btc_status launch_one2(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                              const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  using namespace skinny;
  const int sgs = (d.nchunks + kSG - 1) / kSG;
  const int lds = one_lds_bytes(OneCfg<B>::kE8Bytes, sgs);
  static bool attr_set = false;  // one-time kernel attribute, not call state
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemv_mfma_one_kernel<V, B, R>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            80 * 1024) != hipSuccess)
      return BTC_ERR_HIP;
    attr_set = true;
  }
  gemv_mfma_one_kernel<V, B, R><<<(d.out + 16 * R - 1) / (16 * R), kOneWaves * 64, lds, q>>>(d, packed, codebook, alpha, mu,
                                                                           (const uint16_t*)x, y, y_is_f32);
  return launch_status();
}

// Rows per workgroup: the kernel is written for R blocks of 16, but 16 rows is what the matrices
// it is chosen for want (measured on 4096 x 11008: 8.6 us with 16 rows, 11.3 with 32, 17.8 with 64).
template <int V, int B>
static btc_status launch_one(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                             const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  return launch_one2<V, B, 1>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
}

btc_status gemv_mfma_one(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook,
                         const float* alpha, const float* mu, const void* x, void* y, int y_is_f32) {
  switch (d.v * 16 + d.b) {
    case 10 * 16 + 7: return launch_one<10, 7>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 10 * 16 + 8: return launch_one<10, 8>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 10 * 16 + 9: return launch_one<10, 9>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 10 * 16 + 10: return launch_one<10, 10>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 9 * 16 + 7: return launch_one<9, 7>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 9 * 16 + 8: return launch_one<9, 8>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 9 * 16 + 9: return launch_one<9, 9>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    case 9 * 16 + 10: return launch_one<9, 10>(q, d, packed, codebook, alpha, mu, x, y, y_is_f32);
    default: return BTC_ERR_UNSUPPORTED;
  }
}

bool gemv_mfma_covers(const Dims& d, int batch) {
  return batch >= 1 && batch <= 16 && (d.v == 9 || d.v == 10) && d.b >= 7 && d.b <= 10 && (d.in & 1) == 0 &&
         (long long)d.out * d.wpr * 4 < (1LL << 31) && (long long)batch * d.in * 2 < (1LL << 31);
}

// Workspace of a call: the row sums (one copy per block of the second pass), then the partial sums.
static size_t xpart_bytes(const Dims& d, const skinny::Plan& pl) {
  const int n_rb = (d.out + skinny::kReduceCols - 1) / skinny::kReduceCols;
  return (size_t)n_rb * pl.n_ct * 16 * sizeof(float);
}

size_t gemv_mfma_workspace_bytes(const Dims& d, int batch) {
  const skinny::Plan pl = skinny::make_plan(d);
  return xpart_bytes(d, pl) + (size_t)pl.n_ct * batch * d.out * sizeof(float);
}

// Fitted to measurements on 2 .. 26 MB matrices: launches, prologue and second pass, plus the
// index stream, plus what grows with the number of activation rows (staging, partial sums).
double gemv_mfma_estimate_us(const Dims& d, int batch) {
  const double bytes = (double)d.out * d.wpr * 4;
  return 8.4 + 0.47e-6 * bytes + batch / 16.0 * (1.8 + 0.13e-6 * bytes);
}

btc_status skinny_reduce(hipStream_t q, const float* alpha, const float* mu, float* part, float* xpart, int out,
                         int rows, int n_ct, int xstride, void* y, int y_dtype) {
  const int n_rb = (out + skinny::kReduceCols - 1) / skinny::kReduceCols;
  skinny::skinny_reduce_kernel<<<dim3(n_rb, rows), 256, 0, q>>>(alpha, mu, part, xpart, out, rows, n_ct, xstride, y,
                                                               y_dtype);
  return launch_status();
}

btc_status gemv_mfma(hipStream_t q, const Dims& d, const uint32_t* packed, const uint32_t* codebook, const float* alpha,
                     const float* mu, const void* x, int is_bf16, int batch, void* y, int y_dtype, void* workspace) {
  using namespace skinny;
  const Plan pl = make_plan(d);
  const int n_rb = (d.out + kReduceCols - 1) / kReduceCols;
  float* xpart = (float*)workspace;
  float* part = (float*)((char*)workspace + xpart_bytes(d, pl));
  btc_status st;
  switch (d.v * 16 + d.b) {
    case 10 * 16 + 7: st = launch1<10, 7>(q, d, pl, packed, codebook, x, is_bf16, batch, part, xpart, n_rb); break;
    case 10 * 16 + 8: st = launch1<10, 8>(q, d, pl, packed, codebook, x, is_bf16, batch, part, xpart, n_rb); break;
    case 10 * 16 + 9: st = launch1<10, 9>(q, d, pl, packed, codebook, x, is_bf16, batch, part, xpart, n_rb); break;
    case 10 * 16 + 10: st = launch1<10, 10>(q, d, pl, packed, codebook, x, is_bf16, batch, part, xpart, n_rb); break;
    case 9 * 16 + 7: st = launch1<9, 7>(q, d, pl, packed, codebook, x, is_bf16, batch, part, xpart, n_rb); break;
    case 9 * 16 + 8: st = launch1<9, 8>(q, d, pl, packed, codebook, x, is_bf16, batch, part, xpart, n_rb); break;
    case 9 * 16 + 9: st = launch1<9, 9>(q, d, pl, packed, codebook, x, is_bf16, batch, part, xpart, n_rb); break;
    case 9 * 16 + 10: st = launch1<9, 10>(q, d, pl, packed, codebook, x, is_bf16, batch, part, xpart, n_rb); break;
    default: return BTC_ERR_UNSUPPORTED;
  }
  if (st != BTC_OK) return st;
  return skinny_reduce(q, alpha, mu, part, xpart, d.out, batch, pl.n_ct, 16, y, y_dtype);
}

}  // namespace btc
