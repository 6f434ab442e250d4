// 8-bit weights: a projection matrix is int8 with one fp32 scale per output row, W[n][k] = scale[n] * q[n][k].
// The kernels turn q into bf16 in registers (exact: |q| <= 127 fits the 8 significant bits of bf16), multiply
// on the matrix cores as for 16-bit weights, and multiply the reduced result tile by the column's scale.
//
// Re-tiled layout: 16-row groups of tiles of 16 rows x 64 k (1 KiB); lane l of a tile holds the 16 bytes of row
// l % 16 at k = 16 (l / 16) .. + 16.  One tile feeds two matrix instructions: the first takes bytes 0-7 of every
// lane (k = 16 g + 0..7 for g = 0..3), the second bytes 8-15; the x fragments are gathered with the same k sets.
#pragma once

#include "common.hpp"

namespace sd {

typedef uint32_t q8_u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t q8_u32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 q8_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float q8_f32x2_t __attribute__((ext_vector_type(2)));

// four int8 in a dword -> four bf16 in two dwords (element order kept)
__device__ __forceinline__ q8_u32x2_t q8_dword_to_bf16(uint32_t d) {
    const int32_t s = (int32_t)d;
    const q8_f32x2_t a = {(float)(int8_t)(s), (float)(int8_t)(s >> 8)};
    const q8_f32x2_t b = {(float)(int8_t)(s >> 16), (float)(s >> 24)};
    q8_u32x2_t r;
    r.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, q8_bf16x2_t));
    r.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, q8_bf16x2_t));
    return r;
}

// eight int8 -> one bf16x8 operand
__device__ __forceinline__ q8_u32x4_t q8_half_to_bf16(q8_u32x2_t raw) {
    const q8_u32x2_t lo = q8_dword_to_bf16(raw.x), hi = q8_dword_to_bf16(raw.y);
    return q8_u32x4_t{lo.x, lo.y, hi.x, hi.y};
}

}  // namespace sd
