// Helpers for v_mfma_f32_16x16x32_f16 operands.
//
// Register layout (lane = 16*kb + x, x = lane & 15, kb = lane >> 4):
//   A operand: row x,    k-slots 8*kb .. 8*kb+7 (8 halves in 4 VGPRs)
//   B operand: column x, same k-slots
//   C/D      : column x, rows 4*kb .. 4*kb+3 (4 floats)
// The k-slot -> meaning assignment is free as long as A and B agree, and an
// accumulator tile can feed the next product as an operand without moving data.
#pragma once
#include "vidkv_common.h"

namespace vidkv {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));

union Op {   // one MFMA operand
  h8 v;
  uint32_t u[4];
  h2 p[4];
  u32x4 q;
};

__device__ __forceinline__ f4 mma(const Op& a, const Op& b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.v, b.v, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t h2_bits(h2 x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ h2 bits_h2(uint32_t x) { return __builtin_bit_cast(h2, x); }

// The 8 token slots of a lane group kb inside a 32-token group:
// slot i < 4 -> token 4*kb + i, slot i >= 4 -> token 16 + 4*kb + (i - 4).
__device__ __forceinline__ int slot_token(int kb, int i) {
  return (i < 4) ? 4 * kb + i : 16 + 4 * kb + (i - 4);
}

// cos(2 pi j / 32), j = 0..31, rounded to fp32 (quarter-turn values exact).
static __device__ const float kCosT[32] = {
    cos32(0),  cos32(1),  cos32(2),  cos32(3),  cos32(4),  cos32(5),  cos32(6),  cos32(7),
    cos32(8),  cos32(9),  cos32(10), cos32(11), cos32(12), cos32(13), cos32(14), cos32(15),
    cos32(16), cos32(17), cos32(18), cos32(19), cos32(20), cos32(21), cos32(22), cos32(23),
    cos32(24), cos32(25), cos32(26), cos32(27), cos32(28), cos32(29), cos32(30), cos32(31)};

}  // namespace vidkv
