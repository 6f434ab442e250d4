// Shared device helpers for the gfx950 kernels: bf16 packing, wave reductions, Philox4x32-10.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd {

constexpr int WAVE = 64;

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest even; inputs are finite in this library
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Activations feed the matrix cores as two bf16 terms, v ~= hi + lo (about 16 significant bits): the second
// matrix instruction per tile is free in a weight-streaming kernel and keeps deep models inside the logit
// tolerance.  `lo_off` is the element offset from a buffer's hi half to its lo half (0: no lo half).
__device__ __forceinline__ void store_split_bf16(bf16_t *p, size_t o, int64_t lo_off, float v) {
    const bf16_t hi = f32_to_bf16(v);
    p[o] = hi;
    if (lo_off) p[o + lo_off] = f32_to_bf16(v - bf16_to_f32(hi));
}

template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, WAVE);
    return v;
}
template <typename T> __device__ __forceinline__ T wave_max(T v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        T o = __shfl_xor(v, m, WAVE);
        v = o > v ? o : v;
    }
    return v;
}

// ---- Philox4x32-10 (Salmon et al., SC'11): counter-based, ten rounds ---------------------------
struct Philox4 { uint32_t v[4]; };

__host__ __device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                           uint32_t k0, uint32_t k1) {
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)M0 * c0;
        const uint64_t p1 = (uint64_t)M1 * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    Philox4 o;
    o.v[0] = c0; o.v[1] = c1; o.v[2] = c2; o.v[3] = c3;
    return o;
}

enum { PURPOSE_DRAFT = 0, PURPOSE_ACCEPT = 1, PURPOSE_RESID = 2, PURPOSE_BONUS = 3, PURPOSE_FORCED = 4 };

// 24-bit uniform in [0,1): exact in fp32 and fp64
__host__ __device__ __forceinline__ double philox_uniform(uint64_t seed, uint32_t s, uint32_t i, uint32_t purpose,
                                                          uint32_t b) {
    Philox4 r = philox4x32_10(s, i, purpose, b, (uint32_t)seed, (uint32_t)(seed >> 32));
    return (double)(r.v[0] >> 8) * (1.0 / 16777216.0);
}

}  // namespace sd
