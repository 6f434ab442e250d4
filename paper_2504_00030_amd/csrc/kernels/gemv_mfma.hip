// Weight-streaming projections on the matrix cores for 3..128 rows (the verification pass of a
// speculative step over gamma+1 rows per sequence, and prompt ingestion).
//
// Weights are read from a re-tiled copy: 16-row groups, each a contiguous run of 1 KiB tiles
// (16 rows x 32 k) stored lane-major, so that a wave's 16-byte-per-lane load of one tile is one
// contiguous KiB and IS the B operand of v_mfma_f32_16x16x32_bf16.  The x rows (bf16) are the A
// operand, fetched from L2 with the same 16-byte pattern.  The NW waves of a workgroup split K,
// leave their partial tiles in LDS, the partials are summed in wave order (fixed order: results
// repeat bit for bit), and the epilogue (RoPE + KV write, residual + next-norm statistics, SwiGLU,
// logits + softmax partials) runs on the reduced tile.  The pass stays HBM-bound: one MFMA per KiB
// of weights per 16 rows.
#include <hip/hip_ext.h>

#include "common.hpp"
#include "epilogue.hpp"
#include "kv.hpp"
#include "params.hpp"

namespace sd {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// NG: 16-row groups per workgroup; MB: 16-row blocks of x; NW: waves (K slices) per workgroup.
template <int EPI, int NG, int MB, int NW>
__global__ __launch_bounds__(NW * 64) void gemv_mfma_k(const GemvArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int NT = NW * 64;
    constexpr int FR = MB * NG * 256;   // floats of one wave's partial tile
    constexpr int TS = NG * 16 + 1;     // row stride of the reduced tile
    // k-tiles whose loads are issued together: bounded by the registers of the weight tiles (NG per k-tile) and
    // of the x fragments (hi and lo terms of half a batch for each of the MB row blocks)
    constexpr int UB = NG >= 4 ? 2 : (NG == 2 ? 4 : 8);
    constexpr int UA = 40 / (NG + MB) >= 8 ? 8 : (40 / (NG + MB) >= 4 ? 4 : (40 / (NG + MB) >= 2 ? 2 : 1));
    constexpr int U = UA < UB ? UA : UB;
    static_assert(NW * MB * NG <= 32, "partial tiles must fit 32 KiB of LDS");
    // the wave index is made a scalar so that every branch around a matrix instruction is a scalar
    // branch: v_mfma ignores the execution mask, and a short masked block whose skip branch the compiler
    // drops would run it on undefined operands
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int Ntot = a.n0;
    if (EPI == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (EPI == EPI_SWIGLU) Ntot = 2 * a.n0;
    const int n_groups = Ntot >> 4;
    const int g0 = blockIdx.x * NG;
    const int K = a.K, KT = K >> 5;
    const int KTw = (KT + NW - 1) / NW;
    const int kt_begin = min(wave * KTw, KT), kt_end = min(kt_begin + KTw, KT);
    const int R = a.R;

    __shared__ float part[NW * FR];
    __shared__ float tile[MB * 16 * TS];
    __shared__ float s_scale[MB * 16];

    RowScales<NT> rs;
    rs.begin(a, R);

    const u32x4_t *bp[NG];
#pragma unroll
    for (int ng = 0; ng < NG; ++ng) {
        const int g = min(g0 + ng, n_groups - 1);
        bp[ng] = reinterpret_cast<const u32x4_t *>(a.w0) + ((size_t)g * KT + kt_begin) * 64 + lane;
    }
    // x fragments: lane l holds row 16 mb + l % 16.  Rows at or beyond R produce output rows nobody reads, so
    // their lanes skip the loads.  x enters as two bf16 terms, x = hi + lo.  With at most 8 rows both terms share
    // one fragment (hi rows in 0..7, lo rows in 8..15: one load and one matrix instruction per tile, the two
    // halves of the result are added in the reduction); otherwise the lo term takes a second fragment.
    const bool has_lo = a.xb_lo != 0;            // kernel arguments: scalar conditions
    const bool fold = has_lo && MB == 1 && R <= 8;
    const bool two_terms = has_lo && !fold;
    const u32x4_t *ap[MB];
    bool row_ok[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        int r = mb * 16 + (lane & 15);
        size_t off = 0;
        if (fold && r >= 8) { r -= 8; off = (size_t)a.xb_lo; }
        row_ok[mb] = r < R;
        const size_t xr = (size_t)(min(r, R - 1) * a.x_mul + a.x_add);
        ap[mb] = reinterpret_cast<const u32x4_t *>(a.xb + off + xr * K + (size_t)kt_begin * 32 + (lane >> 4) * 8);
    }
    f32x4_t acc[NG][MB];
#pragma unroll
    for (int ng = 0; ng < NG; ++ng)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[ng][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // One batch = U k-tiles.  The x fragments (short latency: L2) are fetched for half a batch at a time, the
    // first half before the weight loads and the second after the first half's matrix instructions, so that
    // they take half the registers; the weight loads (HBM) of the whole batch are in flight together.
    constexpr int UH = U >= 2 ? U / 2 : 1;
    for (int kt = kt_begin; kt < kt_end; kt += U) {
        u32x4_t bw[U][NG], aw[UH][MB], al[UH][MB];
        auto load_x = [&](int h) {
#pragma unroll
            for (int i = 0; i < UH; ++i) {
                const int u = h * UH + i;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    aw[i][mb] = u32x4_t{0u, 0u, 0u, 0u};
                    al[i][mb] = u32x4_t{0u, 0u, 0u, 0u};
                }
                if (kt + u < kt_end) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        if (row_ok[mb]) {
                            aw[i][mb] = ap[mb][4 * u];
                            if (two_terms)
                                al[i][mb] = *reinterpret_cast<const u32x4_t *>(
                                    reinterpret_cast<const uint16_t *>(ap[mb] + 4 * u) + a.xb_lo);
                        }
                    }
                }
            }
        };
        auto multiply = [&](int h) {
#pragma unroll
            for (int i = 0; i < UH; ++i) {
                const int u = h * UH + i;
                if (kt + u < kt_end) {
#pragma unroll
                    for (int ng = 0; ng < NG; ++ng)
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) {
                            acc[ng][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(bf16x8_t, aw[i][mb]), __builtin_bit_cast(bf16x8_t, bw[u][ng]), acc[ng][mb],
                                0, 0, 0);
                            if (two_terms)
                                acc[ng][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    __builtin_bit_cast(bf16x8_t, al[i][mb]), __builtin_bit_cast(bf16x8_t, bw[u][ng]),
                                    acc[ng][mb], 0, 0, 0);
                        }
                }
            }
        };
        load_x(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kt + u < kt_end) {
#pragma unroll
                for (int ng = 0; ng < NG; ++ng) bw[u][ng] = __builtin_nontemporal_load(bp[ng] + 64 * u);
            }
        }
        multiply(0);
        if (U >= 2) {
            load_x(1);
            multiply(1);
        }
#pragma unroll
        for (int ng = 0; ng < NG; ++ng) bp[ng] += 64 * U;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) ap[mb] += 4 * U;
    }

    // partial tiles -> LDS (register layout: [mb][ng][v][lane])
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int ng = 0; ng < NG; ++ng)
#pragma unroll
            for (int v = 0; v < 4; ++v) part[wave * FR + (((mb * NG + ng) * 4 + v) << 6) + lane] = acc[ng][mb][v];
    __syncthreads();
    // sum the K slices in wave order and lay the result out row-major:
    // register (mb, ng, v, lane) is x row 16 mb + 4 (lane / 16) + v, column 16 ng + lane % 16
    for (int idx = threadIdx.x; idx < FR; idx += NT) {
        float s = part[idx];
#pragma unroll
        for (int w = 1; w < NW; ++w) s += part[w * FR + idx];
        const int l = idx & 63, v = (idx >> 6) & 3, t = idx >> 8;
        if (fold) {
            // rows 8..15 hold the lo term of rows 0..7: lane l + 32 of the same register
            if (l >= 32) continue;
            float s2 = part[idx + 32];
#pragma unroll
            for (int w = 1; w < NW; ++w) s2 += part[w * FR + idx + 32];
            s += s2;
        }
        const int mb = t / NG, ng = t % NG;
        tile[(mb * 16 + (l >> 4) * 4 + v) * TS + ng * 16 + (l & 15)] = s;
    }
    rs.finish(a, s_scale, R);  // ends with a barrier

    if constexpr (EPI == EPI_SWIGLU || EPI == EPI_QKV) {
        // pairs live inside each 16-row group
#pragma unroll
        for (int ng = 0; ng < NG; ++ng)
            if (g0 + ng < n_groups) epilogue_tile<EPI, 16, NT>(a, tile + ng * 16, TS, s_scale, R, g0 + ng, Ntot, threadIdx.x);
    } else {
        epilogue_tile<EPI, NG * 16, NT>(a, tile, TS, s_scale, R, blockIdx.x, Ntot, threadIdx.x);
    }
}

// ---- launch configuration ---------------------------------------------------------------------------
// (NG, NW) by matrix shape and row blocks: enough waves to fill 256 CUs with loads in flight, at least a
// few k-tiles per wave, and NW * MB * NG <= 32 (LDS budget of the partial tiles).
struct MfmaCfg { int ng, nw; };

static MfmaCfg pick_cfg(int n_groups, int KT, int MB, int forced) {
    if (forced > 0) return MfmaCfg{forced / 100, forced % 100};
    // measured on MI355X (plain epilogue, weights rotated through > 2 GiB): one group per workgroup with
    // eight K slices streams fastest while x is a single 16-row block; with more row blocks the x operand
    // traffic grows and tall matrices do better with more groups per workgroup (x fragments reused)
    MfmaCfg c;
    if (MB == 1) c = MfmaCfg{1, 8};
    else if (MB == 2) c = n_groups >= 1024 ? MfmaCfg{4, 4} : (n_groups >= 320 ? MfmaCfg{2, 4} : MfmaCfg{1, 8});
    else if (MB == 4) c = n_groups >= 1024 ? MfmaCfg{2, 4} : MfmaCfg{1, 8};
    else c = MfmaCfg{1, 4};
    while (c.nw > 4 && KT / c.nw < 2) c.nw /= 2;  // keep at least two k-tiles per wave
    return c;
}

int gemv_mfma_groups_per_wg(int epi, int Ntot, int K, int R, int forced) {
    (void)epi;
    const int MB = R <= 16 ? 1 : (R <= 32 ? 2 : (R <= 64 ? 4 : 8));
    return pick_cfg(Ntot / 16, K / 32, MB, forced).ng;
}

// Events of an optional timed launch: recorded by the dispatch itself (start and end of the kernel,
// nothing of the launch path in between).
struct LaunchEvents { hipEvent_t start, stop; };

template <int EPI, int NG, int MB, int NW>
static hipError_t launch_one(const GemvArgs &a, int blocks, LaunchEvents ev, hipStream_t s) {
    if constexpr (NW * MB * NG <= 32) {
        if (ev.start != nullptr)
            hipExtLaunchKernelGGL((gemv_mfma_k<EPI, NG, MB, NW>), dim3(blocks), dim3(NW * 64), 0, s, ev.start, ev.stop, 0, a);
        else
            hipLaunchKernelGGL((gemv_mfma_k<EPI, NG, MB, NW>), dim3(blocks), dim3(NW * 64), 0, s, a);
        return hipGetLastError();
    } else {
        return hipErrorInvalidValue;
    }
}

template <int EPI, int NG, int NW>
static hipError_t launch_mb(const GemvArgs &a, int MB, int blocks, LaunchEvents ev, hipStream_t s) {
    switch (MB) {
        case 1: return launch_one<EPI, NG, 1, NW>(a, blocks, ev, s);
        case 2: return launch_one<EPI, NG, 2, NW>(a, blocks, ev, s);
        case 4: return launch_one<EPI, NG, 4, NW>(a, blocks, ev, s);
        default: return launch_one<EPI, NG, 8, NW>(a, blocks, ev, s);
    }
}

template <int EPI>
static hipError_t launch_cfg(const GemvArgs &a, int Ntot, int forced, LaunchEvents ev, hipStream_t s) {
    const int MB = a.R <= 16 ? 1 : (a.R <= 32 ? 2 : (a.R <= 64 ? 4 : 8));
    const int n_groups = Ntot / 16;
    const MfmaCfg c = pick_cfg(n_groups, a.K / 32, MB, forced);
    const int blocks = (n_groups + c.ng - 1) / c.ng;
    const int key = c.ng * 100 + c.nw;
    switch (key) {
        case 116: return launch_mb<EPI, 1, 16>(a, MB, blocks, ev, s);
        case 108: return launch_mb<EPI, 1, 8>(a, MB, blocks, ev, s);
        case 104: return launch_mb<EPI, 1, 4>(a, MB, blocks, ev, s);
        case 208: return launch_mb<EPI, 2, 8>(a, MB, blocks, ev, s);
        case 204: return launch_mb<EPI, 2, 4>(a, MB, blocks, ev, s);
        case 404: return launch_mb<EPI, 4, 4>(a, MB, blocks, ev, s);
    }
    return hipErrorInvalidValue;
}

// Host-side contract: w0 is the re-tiled matrix (for QKV / SWIGLU the fused, pair-interleaved one),
// Ntot % 16 == 0, K % 32 == 0, xb holds bf16 rows of length K, 1 <= R <= 128;
// RESID: gridDim.x <= ssq_stride; LOGITS: n_tiles == gridDim.x.  `forced` = NG * 100 + NW overrides the
// shape heuristic (0 = automatic).  With ev_start / ev_stop non-null the dispatch records them at the
// kernel's start and end.
hipError_t launch_gemv_mfma(const GemvArgs &a, int epi, int forced, hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t s) {
    const LaunchEvents ev{ev_start, ev_stop};
    int Ntot = a.n0;
    if (epi == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (epi == EPI_SWIGLU) Ntot = 2 * a.n0;
    if (a.R < 1 || a.R > 128 || Ntot % 16 || a.K % 32 || a.xb == nullptr) return hipErrorInvalidValue;
    switch (epi) {
        case EPI_PLAIN: return launch_cfg<EPI_PLAIN>(a, Ntot, forced, ev, s);
        case EPI_QKV: return launch_cfg<EPI_QKV>(a, Ntot, forced, ev, s);
        case EPI_RESID: return launch_cfg<EPI_RESID>(a, Ntot, forced, ev, s);
        case EPI_SWIGLU: return launch_cfg<EPI_SWIGLU>(a, Ntot, forced, ev, s);
        case EPI_LOGITS: return launch_cfg<EPI_LOGITS>(a, Ntot, forced, ev, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace sd
