// Device helpers shared by the kernels that feed table entries straight into MFMA 16x16x32
// operands (btc_gemv_mfma.hip, btc_gemm_rows.hip): operand types, the table geometry per index
// width, the layout of the staged activations.
#pragma once
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <type_traits>
#include <utility>

#include "btc_internal.h"

namespace btc {
namespace skinny {

// f(integral_constant<int, I>) for I = Begin .. End - 1, fully unrolled
template <int Begin, int End, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (Begin < End) {
    f(std::integral_constant<int, Begin>{});
    static_for<Begin + 1, End>(f);
  }
}

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kWaves = 16;               // 1024 threads: one workgroup per compute unit, 128 registers per lane
constexpr int kSG = 64;                 // chunks per super-group
constexpr int kReduceCols = 256;        // outputs per block of the second pass
constexpr int kMaxSG = 4;               // super-groups of activations a workgroup stages
constexpr int kAhead = 1;               // index words are requested this many super-groups ahead of their use
constexpr uint32_t kOob = 0x80000000u;  // buffer offset that is always out of range
constexpr int kRsrcFlags = 0x00020000;

template <int B>
struct Cfg {
  static constexpr int kNW = B <= 8 ? 4 : 5;                              // index words per lane and super-group
  static constexpr int kK2 = 1 << B;
  static constexpr int kRep = (4096 >> B) > 16 ? 16 : (4096 >> B);        // copies of a 16-byte entry
  static constexpr int kE8Bytes = kK2 * kRep * 16;                        // <= 64 KB
};

constexpr int lds_bytes(int e8, int nsg) { return e8 + nsg * kSG * (256 + 64); }

// position (in words) of the 4-byte tail of (chunk c, activation row j): inside a block of 4 chunks
// (64 words = every bank once) the 16-word slot of a chunk is rotated by c / 16, so that the four
// lane groups of a wave, whose chunks are 16 apart, read from different banks.
__device__ __forceinline__ int x2_word(int c, int j) { return (c >> 2) * 64 + (((c & 3) + (c >> 4)) & 3) * 16 + j; }

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

template <bool BF16>
__device__ __forceinline__ f32x4 mfma16(const uint4& a, const uint4& b, const f32x4& c) {
  if constexpr (BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

}  // namespace skinny
}  // namespace btc
