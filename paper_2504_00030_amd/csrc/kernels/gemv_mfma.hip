// Weight-streaming projections on the matrix cores for 3..128 rows (the verification pass of a
// speculative step over gamma+1 rows per sequence, and prompt ingestion).
//
// Weights are read from a re-tiled copy: 16-row groups, each a contiguous run of 1 KiB tiles
// (16 rows x 32 k) stored lane-major, so that a wave's 16-byte-per-lane load of one tile is one
// contiguous KiB and IS the B operand of v_mfma_f32_16x16x32_bf16.  The x rows (bf16) are the A
// operand, fetched from L2 with the same 16-byte pattern.  The four waves of a workgroup split K,
// reduce through LDS in wave order, and the epilogue (RoPE + KV write, residual + next-norm
// statistics, SwiGLU, logits + softmax partials) runs on the reduced tile.  The pass stays
// HBM-bound: one MFMA per KiB of weights per 16 rows.
#include "common.hpp"
#include "kv.hpp"
#include "params.hpp"

namespace sd {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int MF_SLOT_ROWS = 8;   // rows per wave whose norm statistics are prefetched into registers
constexpr int MF_SLOT_REGS = 4;   // x 64 lanes = 256 slots

// Element (row r of the block, column n of the tile) of the reduced accumulator tile in LDS.
// Layout mirrors the MFMA result registers: [tile = mb * NG + ng][v = r % 4][lane = (r % 16 / 4) * 16 + n % 16].
template <int NG>
__device__ __forceinline__ int tile_off(int r, int n) {
    const int mb = r >> 4, i = r & 15, ng = n >> 4, j = n & 15;
    return (((mb * NG + ng) * 4 + (i & 3)) << 6) + ((i >> 2) << 4) + j;
}

template <int EPI, int NG, int MB>
__global__ __launch_bounds__(256) void gemv_mfma_k(const GemvArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int Ntot = a.n0;
    if (EPI == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (EPI == EPI_SWIGLU) Ntot = 2 * a.n0;
    const int n_groups = Ntot >> 4;
    const int g0 = blockIdx.x * NG;
    const int K = a.K, KT = K >> 5;
    const int KTw = (KT + 3) >> 2;
    const int kt_begin = min(wave * KTw, KT), kt_end = min(kt_begin + KTw, KT);
    const int R = a.R;

    __shared__ float tile[MB * NG * 256];
    __shared__ float s_scale[MB * 16];

    // norm statistics of the input rows: loads issued now, reduced after the streaming loop
    const bool normed = a.ssq_in != nullptr;
    const bool early = normed && R <= 4 * MF_SLOT_ROWS && a.ssq_in_slots <= 64 * MF_SLOT_REGS;
    float sl[MF_SLOT_ROWS][MF_SLOT_REGS];
    if (early) {
#pragma unroll
        for (int i = 0; i < MF_SLOT_ROWS; ++i) {
            const int r = wave + 4 * i;
            const int xr = min(r, R - 1) * a.x_mul + a.x_add;
#pragma unroll
            for (int s = 0; s < MF_SLOT_REGS; ++s) {
                const int slot = lane + 64 * s;
                sl[i][s] = (r < R && slot < a.ssq_in_slots) ? a.ssq_in[(size_t)xr * a.ssq_stride + slot] : 0.f;
            }
        }
    }

    const u32x4_t *bp[NG];
#pragma unroll
    for (int ng = 0; ng < NG; ++ng) {
        const int g = min(g0 + ng, n_groups - 1);
        bp[ng] = reinterpret_cast<const u32x4_t *>(a.w0) + ((size_t)g * KT + kt_begin) * 64 + lane;
    }
    const u32x4_t *ap[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int r = min(mb * 16 + (lane & 15), R - 1);
        const size_t xr = (size_t)(r * a.x_mul + a.x_add);
        ap[mb] = reinterpret_cast<const u32x4_t *>(a.xb + xr * K + (size_t)kt_begin * 32 + (lane >> 4) * 8);
    }
    f32x4_t acc[NG][MB];
#pragma unroll
    for (int ng = 0; ng < NG; ++ng)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[ng][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

#pragma unroll 4
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        u32x4_t bw[NG], aw[MB];
#pragma unroll
        for (int ng = 0; ng < NG; ++ng) {
            bw[ng] = __builtin_nontemporal_load(bp[ng]);
            bp[ng] += 64;
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            aw[mb] = *ap[mb];
            ap[mb] += 4;
        }
#pragma unroll
        for (int ng = 0; ng < NG; ++ng)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                acc[ng][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, aw[mb]),
                                                                     __builtin_bit_cast(bf16x8_t, bw[ng]), acc[ng][mb],
                                                                     0, 0, 0);
    }

    // reduce the four K slices in wave order (fixed order: results repeat bit for bit)
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int ng = 0; ng < NG; ++ng)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int o = (((mb * NG + ng) * 4 + v) << 6) + lane;
                        tile[o] = (w == 0) ? acc[ng][mb][v] : tile[o] + acc[ng][mb][v];
                    }
        }
        __syncthreads();
    }

    // row scales rsqrt(mean(x^2) + eps)
    if (normed) {
        if (early) {
#pragma unroll
            for (int i = 0; i < MF_SLOT_ROWS; ++i) {
                const int r = wave + 4 * i;
                float s = 0.f;
#pragma unroll
                for (int q = 0; q < MF_SLOT_REGS; ++q) s += sl[i][q];
                s = wave_sum(s);
                if (lane == 0 && r < R) s_scale[r] = rsqrtf(s / (float)K + a.eps);
            }
        } else {
            for (int r = wave; r < R; r += 4) {
                const int xr = r * a.x_mul + a.x_add;
                float s = 0.f;
                for (int slot = lane; slot < a.ssq_in_slots; slot += 64) s += a.ssq_in[(size_t)xr * a.ssq_stride + slot];
                s = wave_sum(s);
                if (lane == 0) s_scale[r] = rsqrtf(s / (float)K + a.eps);
            }
        }
    } else {
        for (int r = threadIdx.x; r < R; r += 256) s_scale[r] = 1.f;
    }
    __syncthreads();

    constexpr int NC = NG * 16;  // columns of the tile
    const int n_base = g0 * 16;
    if constexpr (EPI == EPI_PLAIN) {
        for (int idx = threadIdx.x; idx < R * NC; idx += 256) {
            const int r = idx / NC, c = idx % NC;
            if (n_base + c < Ntot) a.y[(size_t)r * a.n0 + n_base + c] = tile[tile_off<NG>(r, c)] * s_scale[r];
        }
    } else if constexpr (EPI == EPI_RESID) {
        const int total = ((R * NC + 255) / 256) * 256;
        for (int idx = threadIdx.x; idx < total; idx += 256) {
            const int r = idx / NC, c = idx % NC;
            const int n = n_base + c;
            float sq = 0.f;
            if (r < R && n < Ntot) {
                const size_t o = (size_t)r * a.n0 + n;
                const float gn = a.g_next != nullptr ? a.g_next[n] : 1.f;
                const float xn = a.xres[o] + tile[tile_off<NG>(r, c)] * s_scale[r];
                a.xres[o] = xn;
                a.xg[o] = xn * gn;
                a.xgb[o] = f32_to_bf16(xn * gn);
                sq = xn * xn;
            }
#pragma unroll
            for (int m = NC / 2; m >= 1; m >>= 1) sq += __shfl_xor(sq, m, WAVE);
            if (c == 0 && r < R) a.ssq_out[(size_t)r * a.ssq_stride + blockIdx.x] = sq;
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        constexpr int NP = NG * 8;
        for (int idx = threadIdx.x; idx < R * NP; idx += 256) {
            const int r = idx / NP, p = idx % NP;
            const int ng = p >> 3, pj = p & 7;
            const int j = (g0 + ng) * 8 + pj;
            if (j < a.n0) {
                const float gt = tile[tile_off<NG>(r, ng * 16 + pj)] * s_scale[r];
                const float up = tile[tile_off<NG>(r, ng * 16 + 8 + pj)] * s_scale[r];
                const float v = gt / (1.f + __expf(-gt)) * up;
                const size_t o = (size_t)r * a.n0 + j;
                a.y[o] = v;
                a.yb[o] = f32_to_bf16(v);
            }
        }
    } else if constexpr (EPI == EPI_QKV) {
        constexpr int NP = NG * 8;
        const int half = a.hd >> 1;
        for (int idx = threadIdx.x; idx < R * NP; idx += 256) {
            const int r = idx / NP, p = idx % NP;
            const int ng = p >> 3, pj = p & 7;
            const int P = (g0 + ng) * 8 + pj;
            if (P >= (Ntot >> 1)) continue;
            int hh = P / half;
            const int j = P % half;
            float y1 = tile[tile_off<NG>(r, ng * 16 + pj)] * s_scale[r];
            float y2 = tile[tile_off<NG>(r, ng * 16 + 8 + pj)] * s_scale[r];
            const int pos = a.row_pos[r];
            if (hh < a.nq + a.nkv) {
                const float c = a.rope_cos[(size_t)pos * half + j];
                const float s = a.rope_sin[(size_t)pos * half + j];
                const float r1 = y1 * c - y2 * s;
                const float r2 = y2 * c + y1 * s;
                y1 = r1; y2 = r2;
            }
            if (hh < a.nq) {
                float *q = a.y + (size_t)r * a.nq * a.hd + (size_t)hh * a.hd + j;
                q[0] = y1;
                q[half] = y2;
                uint16_t *qb = a.yb + (size_t)r * a.nq * a.hd + (size_t)hh * a.hd + j;
                qb[0] = f32_to_bf16(y1);
                qb[half] = f32_to_bf16(y2);
            } else {
                const bool is_k = hh < a.nq + a.nkv;
                const int kvh = hh - a.nq - (is_k ? 0 : a.nkv);
                const int seq = a.row_seq[r];
                kv_store(a.kv, a.kv_dtype, is_k, seq, pos, kvh, j, y1);
                kv_store(a.kv, a.kv_dtype, is_k, seq, pos, kvh, j + half, y2);
            }
        }
    } else if constexpr (EPI == EPI_LOGITS) {
        const int total = ((R * NC + 255) / 256) * 256;
        for (int idx = threadIdx.x; idx < total; idx += 256) {
            const int r = idx / NC, c = idx % NC;
            const int n = n_base + c;
            const bool valid = r < R && n < Ntot;
            const int orow = min(r, R - 1) * a.y_mul + a.y_add;
            const float v = valid ? tile[tile_off<NG>(min(r, R - 1), c)] * s_scale[min(r, R - 1)] : -INFINITY;
            if (valid) a.y[(size_t)orow * a.y_stride + n] = v;
            float m = v;
            int arg = valid ? n : 0x7fffffff;
#pragma unroll
            for (int msk = NC / 2; msk >= 1; msk >>= 1) {
                const float om = __shfl_xor(m, msk, WAVE);
                const int oa = __shfl_xor(arg, msk, WAVE);
                if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
            }
            double e = valid ? exp((double)(v - m) * (double)a.inv_t) : 0.0;
#pragma unroll
            for (int msk = NC / 2; msk >= 1; msk >>= 1) e += __shfl_xor(e, msk, WAVE);
            if (c == 0 && r < R) {
                const size_t pi = (size_t)orow * a.n_tiles + blockIdx.x;
                a.pm[pi] = m;
                a.ps[pi] = e;
                a.pa[pi] = arg;
            }
        }
    }
}

// 16-row groups per workgroup: more for tall matrices (fewer, fatter workgroups), one for short ones
static int pick_ng(int n_groups) { return n_groups >= 2048 ? 4 : (n_groups >= 1024 ? 2 : 1); }

int gemv_mfma_groups_per_wg(int epi, int Ntot) { (void)epi; return pick_ng(Ntot / 16); }

template <int EPI, int NG>
static hipError_t launch_mb(const GemvArgs &a, int blocks, hipStream_t s) {
    const int MB = (a.R + 15) / 16;
    if (MB <= 1) hipLaunchKernelGGL((gemv_mfma_k<EPI, NG, 1>), dim3(blocks), dim3(256), 0, s, a);
    else if (MB <= 2) hipLaunchKernelGGL((gemv_mfma_k<EPI, NG, 2>), dim3(blocks), dim3(256), 0, s, a);
    else if (MB <= 4) hipLaunchKernelGGL((gemv_mfma_k<EPI, NG, 4>), dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((gemv_mfma_k<EPI, NG, 8>), dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <int EPI>
static hipError_t launch_ng(const GemvArgs &a, int Ntot, hipStream_t s) {
    const int n_groups = Ntot / 16;
    const int NG = pick_ng(n_groups);
    const int blocks = (n_groups + NG - 1) / NG;
    if (NG == 4) return launch_mb<EPI, 4>(a, blocks, s);
    if (NG == 2) return launch_mb<EPI, 2>(a, blocks, s);
    return launch_mb<EPI, 1>(a, blocks, s);
}

// Host-side contract: w0 is the re-tiled matrix (for QKV / SWIGLU the fused, pair-interleaved one),
// Ntot % 16 == 0, K % 32 == 0, xb holds bf16 rows of length K, 1 <= R <= 128;
// RESID: gridDim.x <= ssq_stride; LOGITS: n_tiles == gridDim.x.
hipError_t launch_gemv_mfma(const GemvArgs &a, int epi, hipStream_t s) {
    int Ntot = a.n0;
    if (epi == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (epi == EPI_SWIGLU) Ntot = 2 * a.n0;
    if (a.R < 1 || a.R > 128 || Ntot % 16 || a.K % 32 || a.xb == nullptr) return hipErrorInvalidValue;
    switch (epi) {
        case EPI_PLAIN: return launch_ng<EPI_PLAIN>(a, Ntot, s);
        case EPI_QKV: return launch_ng<EPI_QKV>(a, Ntot, s);
        case EPI_RESID: return launch_ng<EPI_RESID>(a, Ntot, s);
        case EPI_SWIGLU: return launch_ng<EPI_SWIGLU>(a, Ntot, s);
        case EPI_LOGITS: return launch_ng<EPI_LOGITS>(a, Ntot, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace sd
