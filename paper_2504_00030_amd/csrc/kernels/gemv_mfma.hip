// Weight-streaming projections on the matrix cores, 1..128 rows of x (draft decode and the verification
// pass of a speculative step over gamma+1 rows per sequence).
//
// Weights are read from a re-tiled copy: 16-row groups, each a contiguous run of 1 KiB tiles
// (16 rows x 32 k) stored lane-major, so that a wave's 16-byte-per-lane load of one tile is one
// contiguous KiB and IS the B operand of v_mfma_f32_16x16x32_bf16.  The x rows are the A operand, as
// two bf16 terms (x = hi + lo, about 16 significant bits; one bf16 term left a 32-layer model outside the
// logit tolerance).  The waves of a workgroup split K, leave their partial tiles in LDS, the partials
// are summed in wave order (fixed order: results repeat bit for bit), and the epilogue (RoPE + KV
// write, residual + next-norm statistics, SwiGLU, logits + softmax partials) runs on the reduced tile.
// Both kernels stay HBM-bound: one or two matrix instructions per KiB of weights per 16 rows.
//
//   gemv_mfma_k     one workgroup per NG groups, any row count: x fragments re-read per workgroup
//   gemv_persist_k  up to 16 rows: 16-wave workgroups walk the groups with the x fragments resident
//   gemv_q8_k       8-bit weights (q8.hpp: int8 + per-row scale, bf16 in registers) at the shapes the persistent
//                   kernel's 8-bit form does not take
// From a few dozen rows on the dense-contraction kernel (gemm_mfma.hip) is the faster one; the host picks.
#include <hip/hip_ext.h>

#include <cstdlib>

#include "common.hpp"
#include "epilogue.hpp"
#include "kv.hpp"
#include "params.hpp"
#include "q8.hpp"

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
    if constexpr (NG == 1 && MB == 1 && NW <= 8) {  // 16 waves leave 128 registers per lane: too few for two batches
        // One group per workgroup and one row block (the K = 14336 down projection of a decode or verification
        // pass): the registers allow two batches of weight tiles, so the next batch is requested before this one's
        // matrix instructions and the stream does not pause for a load latency per batch.  The x fragments of the
        // whole batch go out before those requests (waiting for a younger load would wait for them too).
        u32x4_t bwA[U], bwB[U];
        auto load_w = [&](u32x4_t(&bw)[U], int kt) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (kt + u < kt_end) bw[u] = __builtin_nontemporal_load(bp[0] + 64 * (kt - kt_begin + u));
        };
        auto batch = [&](const u32x4_t(&bw)[U], u32x4_t(&next)[U], int kt) {
            u32x4_t aw[U], al[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                aw[u] = u32x4_t{0u, 0u, 0u, 0u};
                al[u] = u32x4_t{0u, 0u, 0u, 0u};
                if (kt + u < kt_end && row_ok[0]) {
                    const u32x4_t *xp = ap[0] + 4 * (kt - kt_begin + u);
                    aw[u] = *xp;
                    if (two_terms) al[u] = *reinterpret_cast<const u32x4_t *>(reinterpret_cast<const uint16_t *>(xp) + a.xb_lo);
                }
            }
            load_w(next, kt + U);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (kt + u < kt_end) {
                    acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, aw[u]),
                                                                        __builtin_bit_cast(bf16x8_t, bw[u]), acc[0][0], 0, 0, 0);
                    if (two_terms)
                        acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, al[u]),
                                                                            __builtin_bit_cast(bf16x8_t, bw[u]), acc[0][0], 0, 0, 0);
                }
            }
        };
        load_w(bwA, kt_begin);
        for (int kt = kt_begin; kt < kt_end; kt += 2 * U) {
            batch(bwA, bwB, kt);
            if (kt + U < kt_end) batch(bwB, bwA, kt + U);
        }
    } else
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

// ---- persistent variant for one 16-row block of x -------------------------------------------------
// One workgroup of 16 waves per compute unit walks the groups b, b + G, b + 2G, ...  Wave w multiplies the
// k-tiles w, w + 16, w + 32, ... of every group (the workgroup's 16 loads of one step are 16 consecutive KiB),
// so its x fragments do not depend on the group: they are loaded once and stay in registers.  That removes the
// x traffic of the kernel above, where every workgroup re-reads its x rows (measured: it costs about as much as
// a quarter of the weight stream at 9 rows with both bf16 terms).  After the matrix instructions of a group the
// wave issues the first loads of the next group, which are then in flight while the workgroup sums the partial
// tiles and runs the epilogue; the barriers wait on LDS only, not on those loads.
//   KTW: k-tiles per wave (K = 512 KTW); TERMS: 1 = x as one fragment (single bf16 term, or both terms folded
//   into rows 0-7 / 8-15 for up to 8 rows), 2 = hi and lo fragments.
constexpr int PW = 16;  // waves

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

//   WQ: 1 = 8-bit weights (q8.hpp): a tile spans 64 k and feeds two matrix instructions, so a wave holds KTW x
//   fragments for KTW / 2 tiles.
//   RAG: 1 = K is not a multiple of 512 (the 768-wide draft models): the last round of k-tiles exists only for the
//   first waves; the test is on the scalar wave index, so every branch around a matrix instruction stays scalar.
constexpr int persist_burst(int tpw, int frags) {
    // tiles per burst of loads: a divisor of the wave's tiles per group, at most 8 KiB per wave, 4 KiB where the x
    // fragments already take 64 registers and 2 KiB where they take 80 (a deeper burst there spills)
    const int cap = frags >= 20 ? 2 : (frags >= 16 ? 4 : 8);
    int ub = 1;
    for (int d = 1; d <= cap; ++d)
        if (tpw % d == 0) ub = d;
    return ub;
}

template <int EPI, int KTW, int TERMS, int WQ, int RAG>
__global__ __launch_bounds__(PW * 64) void gemv_persist_k(const GemvArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int NT = PW * 64;
    constexpr int TPW = KTW >> WQ;         // weight tiles per wave and group
    constexpr int UB = persist_burst(TPW, KTW * TERMS);
    constexpr int NB = TPW / UB;           // bursts per group
    static_assert(TPW % UB == 0, "bursts tile the wave's k-tiles");
    static_assert(!(RAG && WQ), "8-bit weights come in whole rounds");
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int Ntot = a.n0;
    if (EPI == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (EPI == EPI_SWIGLU) Ntot = 2 * a.n0;
    const int n_groups = Ntot >> 4;
    const int G = gridDim.x, b = blockIdx.x;
    const int n_my = (n_groups - b + G - 1) / G;  // host: G <= n_groups
    const int K = a.K, KT = K >> (5 + WQ);        // tiles per group; host: PW * (TPW - 1) < KT <= PW * TPW, == unless RAG
    const int R = a.R;
    // tile j of this wave exists (always, unless K leaves the last round short)
    auto live = [&](int j) { return !RAG || wave + PW * j < KT; };

    __shared__ float part[PW * 256];
    __shared__ float tile[16 * 17];
    __shared__ float s_scale[16];

    RowScales<NT, 1> rs;  // 16 waves, at most 16 rows: one row per wave
    rs.begin(a, R);

    // x fragments, once
    const bool fold = TERMS == 1 && a.xb_lo != 0;  // host: then R <= 8
    u32x4_t xh[KTW], xl[TERMS == 2 ? KTW : 1];
    {
        int r = lane & 15;
        size_t off = 0;
        if (fold && r >= 8) { r -= 8; off = (size_t)a.xb_lo; }
        const bool row_ok = r < R;
        const size_t xr = (size_t)(min(r, R - 1) * a.x_mul + a.x_add);
        // fragment j: 16-bit weights, k-tile wave + 16 j, k-chunk lane / 16 of 8; 8-bit weights, tile wave + 16 (j / 2),
        // k-chunk lane / 16 of 16, its first or second 8 columns
        const uint16_t *xp = a.xb + off + xr * K + (size_t)wave * (32 << WQ) + (lane >> 4) * (8 << WQ);
#pragma unroll
        for (int j = 0; j < KTW; ++j) {
            xh[j] = u32x4_t{0u, 0u, 0u, 0u};
            if (TERMS == 2) xl[j] = u32x4_t{0u, 0u, 0u, 0u};
            const size_t ko = WQ ? (size_t)(j >> 1) * PW * 64 + (j & 1) * 8 : (size_t)j * PW * 32;
            if (row_ok && live(j)) {
                xh[j] = *reinterpret_cast<const u32x4_t *>(xp + ko);
                if (TERMS == 2) xl[j] = *reinterpret_cast<const u32x4_t *>(xp + a.xb_lo + ko);
            }
        }
    }
    // weight tiles: group g, k-tile (wave + 16 j) at ((g KT + wave + 16 j) 64 + lane) 16 bytes
    const u32x4_t *wp = reinterpret_cast<const u32x4_t *>(a.w0) + ((size_t)b * KT + wave) * 64 + lane;
    const size_t gstride = (size_t)G * KT * 64;  // in 16-byte units, between two groups of this workgroup
    u32x4_t bw[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u)
        if (live(u)) bw[u] = __builtin_nontemporal_load(wp + (size_t)u * PW * 64);

    // what the residual / QKV epilogues read besides the tile is fetched ahead of the matrix instructions (these
    // loads are older than the next group's weight loads, so waiting for them does not drain the stream)
    constexpr bool PRE = EPI == EPI_RESID || EPI == EPI_QKV;
    EpiPre pre{};
    if constexpr (PRE) epi_prefetch_rows<EPI>(a, R, threadIdx.x, pre);

    for (int i = 0; i < n_my; ++i) {
        if constexpr (PRE) epi_prefetch_group<EPI>(a, R, b + i * G, Ntot, threadIdx.x, pre);
        // 8-bit weights: the scale of this thread's column of the reduced tile, fetched ahead like the operands above
        float wsc = 1.f;
        if (WQ && threadIdx.x < 256) wsc = a.wscale[(size_t)(b + i * G) * 16 + (lane & 15)];
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int t = nb * UB + u;
                if constexpr (WQ == 0) {
                    if (live(t)) {
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xh[t]),
                                                                      __builtin_bit_cast(bf16x8_t, bw[u]), acc, 0, 0, 0);
                        if (TERMS == 2)
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xl[t]),
                                                                          __builtin_bit_cast(bf16x8_t, bw[u]), acc, 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const u32x4_t wb = q8_half_to_bf16(h == 0 ? q8_u32x2_t{bw[u].x, bw[u].y} : q8_u32x2_t{bw[u].z, bw[u].w});
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xh[2 * t + h]),
                                                                      __builtin_bit_cast(bf16x8_t, wb), acc, 0, 0, 0);
                        if (TERMS == 2)
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xl[2 * t + h]),
                                                                          __builtin_bit_cast(bf16x8_t, wb), acc, 0, 0, 0);
                    }
                }
            }
            // next burst: the rest of this group, or the head of the next one
            if (nb + 1 < NB) {
#pragma unroll
                for (int u = 0; u < UB; ++u)
                    if (live((nb + 1) * UB + u)) bw[u] = __builtin_nontemporal_load(wp + (size_t)((nb + 1) * UB + u) * PW * 64);
            } else if (i + 1 < n_my) {
#pragma unroll
                for (int u = 0; u < UB; ++u)
                    if (live(u)) bw[u] = __builtin_nontemporal_load(wp + gstride + (size_t)u * PW * 64);
            }
        }
        wp += gstride;
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave * 256 + v * 64 + lane] = acc[v];
        if (i == 0) rs.finish(a, s_scale, R);  // row scales, once (ends with a full barrier)
        lds_barrier();
        // sum the K slices in wave order; register (v, lane) is x row 4 (lane / 16) + v, column lane % 16
        if (threadIdx.x < 256) {
            const int idx = threadIdx.x, l = idx & 63, v = idx >> 6;
            if (!fold || l < 32) {
                float s = part[idx];
#pragma unroll
                for (int w = 1; w < PW; ++w) s += part[w * 256 + idx];
                if (fold) {
                    // rows 8..15 hold the lo term of rows 0..7: lane l + 32 of the same register
                    float s2 = part[idx + 32];
#pragma unroll
                    for (int w = 1; w < PW; ++w) s2 += part[w * 256 + idx + 32];
                    s += s2;
                }
                tile[((l >> 4) * 4 + v) * 17 + (l & 15)] = WQ ? s * wsc : s;
            }
        }
        lds_barrier();
        if constexpr (PRE) epilogue_tile_pre<EPI>(a, tile, 17, s_scale, R, b + i * G, Ntot, threadIdx.x, pre);
        else epilogue_tile<EPI, 16, NT>(a, tile, 17, s_scale, R, b + i * G, Ntot, threadIdx.x);
    }
}

// ---- persistent variant for 17 to 64 rows --------------------------------------------------------------------
// The same walk over the groups with the x fragments of MB 16-row blocks resident: MB x KTW x TERMS fragments of
// four registers each, at most 16 of them, so K <= 2048 for up to 32 rows and K <= 1024 for up to 64 (the draft
// models' projections when a batch of 17 to 64 sequences decodes in lock-step).  Every weight tile meets MB x TERMS
// matrix instructions; the epilogues are the general ones (any row count), run on the reduced MB x 16-row tile.
template <int EPI, int KTW, int MB, int TERMS, int RAG>
__global__ __launch_bounds__(PW * 64) void gemv_persist_mb_k(const GemvArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int NT = PW * 64;
    constexpr int UB = persist_burst(KTW, 16);
    constexpr int NB = KTW / UB;
    constexpr int FR = MB * 256;  // floats of one wave's partial tile
    static_assert(MB * KTW * TERMS <= 16 && MB >= 2 && MB <= 4, "x fragments must fit 64 registers");
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int Ntot = a.n0;
    if (EPI == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (EPI == EPI_SWIGLU) Ntot = 2 * a.n0;
    const int n_groups = Ntot >> 4;
    const int G = gridDim.x, b = blockIdx.x;
    const int n_my = (n_groups - b + G - 1) / G;  // host: G <= n_groups
    const int K = a.K, KT = K >> 5;               // host: PW (KTW - 1) < KT <= PW KTW, == unless RAG
    const int R = a.R;
    auto live = [&](int t) { return !RAG || wave + PW * t < KT; };

    __shared__ float part[PW * FR];
    __shared__ float tile[MB * 16 * 17];
    __shared__ float s_scale[MB * 16];

    RowScales<NT, MB> rs;  // 16 waves, rows wave, wave + 16, ...
    rs.begin(a, R);

    u32x4_t xh[MB][KTW], xl[TERMS == 2 ? MB : 1][TERMS == 2 ? KTW : 1];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int r = mb * 16 + (lane & 15);
        const bool row_ok = r < R;
        const size_t xr = (size_t)(min(r, R - 1) * a.x_mul + a.x_add);
        const uint16_t *xp = a.xb + xr * K + (size_t)wave * 32 + (lane >> 4) * 8;
#pragma unroll
        for (int t = 0; t < KTW; ++t) {
            xh[mb][t] = u32x4_t{0u, 0u, 0u, 0u};
            if (TERMS == 2) xl[mb][t] = u32x4_t{0u, 0u, 0u, 0u};
            if (row_ok && live(t)) {
                xh[mb][t] = *reinterpret_cast<const u32x4_t *>(xp + (size_t)t * PW * 32);
                if (TERMS == 2) xl[mb][t] = *reinterpret_cast<const u32x4_t *>(xp + a.xb_lo + (size_t)t * PW * 32);
            }
        }
    }
    const u32x4_t *wp = reinterpret_cast<const u32x4_t *>(a.w0) + ((size_t)b * KT + wave) * 64 + lane;
    const size_t gstride = (size_t)G * KT * 64;
    u32x4_t bw[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u)
        if (live(u)) bw[u] = __builtin_nontemporal_load(wp + (size_t)u * PW * 64);

    for (int i = 0; i < n_my; ++i) {
        f32x4_t acc[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int t = nb * UB + u;
                if (live(t)) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xh[mb][t]),
                                                                          __builtin_bit_cast(bf16x8_t, bw[u]), acc[mb], 0, 0, 0);
                        if (TERMS == 2)
                            acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xl[mb][t]),
                                                                              __builtin_bit_cast(bf16x8_t, bw[u]), acc[mb], 0, 0, 0);
                    }
                }
            }
            if (nb + 1 < NB) {
#pragma unroll
                for (int u = 0; u < UB; ++u)
                    if (live((nb + 1) * UB + u)) bw[u] = __builtin_nontemporal_load(wp + (size_t)((nb + 1) * UB + u) * PW * 64);
            } else if (i + 1 < n_my) {
#pragma unroll
                for (int u = 0; u < UB; ++u)
                    if (live(u)) bw[u] = __builtin_nontemporal_load(wp + gstride + (size_t)u * PW * 64);
            }
        }
        wp += gstride;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 4; ++v) part[wave * FR + ((mb * 4 + v) << 6) + lane] = acc[mb][v];
        if (i == 0) rs.finish(a, s_scale, R);  // row scales, once (ends with a full barrier)
        lds_barrier();
        // sum the K slices in wave order; register (mb, v, lane) is x row 16 mb + 4 (lane / 16) + v, column lane % 16
        if (threadIdx.x < FR) {
            const int idx = threadIdx.x, l = idx & 63, v = (idx >> 6) & 3, mb = idx >> 8;
            float sum = part[idx];
#pragma unroll
            for (int w = 1; w < PW; ++w) sum += part[w * FR + idx];
            tile[(mb * 16 + (l >> 4) * 4 + v) * 17 + (l & 15)] = sum;
        }
        lds_barrier();
        epilogue_tile<EPI, 16, NT>(a, tile, 17, s_scale, R, b + i * G, Ntot, threadIdx.x);
    }
}

// ---- K shared out over workgroups, x resident ---------------------------------------------------------------
// The projections whose K is too long for the persistent kernel's registers (the down projections: K = 11008,
// 13824, 14336) and those with fewer groups than half the compute units (K = 8192 of the 1B-shaped draft).  The K
// of every group is cut into S slices; workgroup (s, j) keeps the x fragments of slice s in registers and walks the
// groups j, j + J, ... like the persistent kernel, leaving one partial tile per group in global memory.  The
// workgroup that arrives last at the counter of its set j sums the S partial tiles of each of the set's groups in
// slice order (a fixed order: results repeat bit for bit whoever is last) and runs the epilogue.  Partial tiles and
// counters cross workgroups - and the chip's eight L2s - as agent-scope stores, loads and atomics; nothing is
// fenced (measured on the chip: an arrival through such a counter costs about 2 us, a cache write-back and
// invalidate at agent scope about 5).
//   KTW: k-tiles per wave and slice; RAG: the slice's last round of k-tiles exists only for the first waves.
template <int EPI, int KTW, int TERMS, int RAG>
__global__ __launch_bounds__(PW * 64) void gemv_ksplit_k(const GemvArgs a, const int S) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int UB = persist_burst(KTW, KTW * TERMS);
    constexpr int NB = KTW / UB;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int Ntot = a.n0;
    if (EPI == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (EPI == EPI_SWIGLU) Ntot = 2 * a.n0;
    const int n_groups = Ntot >> 4;
    const int J = gridDim.x / S, s = blockIdx.x % S, j = blockIdx.x / S;   // host: gridDim.x == S * J, J <= n_groups
    const int n_my = (n_groups - j + J - 1) / J;
    const int K = a.K, KT = K >> 5, KTs = KT / S;                          // host: KT % S == 0, PW (KTW - 1) < KTs <= PW KTW
    const int R = a.R;
    auto live = [&](int t) { return !RAG || wave + PW * t < KTs; };

    __shared__ float part[PW * 256];
    __shared__ float s_scale[16];
    __shared__ int s_last;

    RowScales<PW * 64, 1> rs;  // only the workgroup that finishes a set uses them; the loads are cheap and early
    rs.begin(a, R);

    const bool fold = TERMS == 1 && a.xb_lo != 0;  // host: then R <= 8
    u32x4_t xh[KTW], xl[TERMS == 2 ? KTW : 1];
    {
        int r = lane & 15;
        size_t off = 0;
        if (fold && r >= 8) { r -= 8; off = (size_t)a.xb_lo; }
        const bool row_ok = r < R;
        const size_t xr = (size_t)(min(r, R - 1) * a.x_mul + a.x_add);
        const uint16_t *xp = a.xb + off + xr * K + ((size_t)s * KTs + wave) * 32 + (lane >> 4) * 8;
#pragma unroll
        for (int t = 0; t < KTW; ++t) {
            xh[t] = u32x4_t{0u, 0u, 0u, 0u};
            if (TERMS == 2) xl[t] = u32x4_t{0u, 0u, 0u, 0u};
            if (row_ok && live(t)) {
                xh[t] = *reinterpret_cast<const u32x4_t *>(xp + (size_t)t * PW * 32);
                if (TERMS == 2) xl[t] = *reinterpret_cast<const u32x4_t *>(xp + a.xb_lo + (size_t)t * PW * 32);
            }
        }
    }
    const u32x4_t *wp = reinterpret_cast<const u32x4_t *>(a.w0) + ((size_t)j * KT + (size_t)s * KTs + wave) * 64 + lane;
    const size_t gstride = (size_t)J * KT * 64;
    u32x4_t bw[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u)
        if (live(u)) bw[u] = __builtin_nontemporal_load(wp + (size_t)u * PW * 64);

    for (int i = 0; i < n_my; ++i) {
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int t = nb * UB + u;
                if (live(t)) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xh[t]),
                                                                  __builtin_bit_cast(bf16x8_t, bw[u]), acc, 0, 0, 0);
                    if (TERMS == 2)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xl[t]),
                                                                      __builtin_bit_cast(bf16x8_t, bw[u]), acc, 0, 0, 0);
                }
            }
            if (nb + 1 < NB) {
#pragma unroll
                for (int u = 0; u < UB; ++u)
                    if (live((nb + 1) * UB + u)) bw[u] = __builtin_nontemporal_load(wp + (size_t)((nb + 1) * UB + u) * PW * 64);
            } else if (i + 1 < n_my) {
#pragma unroll
                for (int u = 0; u < UB; ++u)
                    if (live(u)) bw[u] = __builtin_nontemporal_load(wp + gstride + (size_t)u * PW * 64);
            }
        }
        wp += gstride;
        lds_barrier();  // the previous group's partials have been read
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave * 256 + v * 64 + lane] = acc[v];
        if (i == 0) rs.finish(a, s_scale, R);  // row scales, once (ends with a full barrier)
        lds_barrier();
        // this slice's tile: the waves' partials in wave order, to global memory as [row][column]
        if (threadIdx.x < 256) {
            const int idx = threadIdx.x, l = idx & 63, v = idx >> 6;
            if (!fold || l < 32) {
                float sum = part[idx];
#pragma unroll
                for (int w = 1; w < PW; ++w) sum += part[w * 256 + idx];
                if (fold) {
                    float s2 = part[idx + 32];
#pragma unroll
                    for (int w = 1; w < PW; ++w) s2 += part[w * 256 + idx + 32];
                    sum += s2;
                }
                const int row = (l >> 4) * 4 + v, col = l & 15;
                if (row < R)
                    __hip_atomic_store(a.ks_part + ((size_t)s * n_groups + (j + i * J)) * 256 + row * 16 + col, sum,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    __syncthreads();  // every store of this workgroup has been acknowledged
    if (threadIdx.x == 0) {
        const uint32_t old = __hip_atomic_fetch_add(a.ks_ticket + j, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = old == (uint32_t)(S - 1);
        if (s_last) __hip_atomic_store(a.ks_ticket + j, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next launch
    }
    __syncthreads();
    if (!s_last) return;
    // Four groups at a time, 256 threads each (thread -> row, column of the group's tile): what the epilogue reads
    // besides the tile goes out first, then the S partial tiles, all groups' loads in flight together.
    const int q = threadIdx.x >> 8, tl = threadIdx.x & 255;
    float *my_tile = part + q * (16 * 17);  // the partials' LDS is free now
    constexpr bool PRE = EPI == EPI_RESID || EPI == EPI_QKV;
    EpiPre pre{};
    if constexpr (EPI == EPI_QKV) epi_prefetch_rows<EPI>(a, R, tl, pre);
    for (int base = 0; base < n_my; base += 4) {
        const int i = base + q;
        const bool mine = i < n_my;  // the same for the four waves of a quarter
        const int g = j + i * J;
        const int row = tl >> 4, col = tl & 15;
        if (mine) {
            if constexpr (PRE) epi_prefetch_group<EPI>(a, R, g, Ntot, tl, pre);
            float sum = 0.f;
            if (row < R) {
                float v[KSPLIT_MAX];
#pragma unroll
                for (int ss = 0; ss < KSPLIT_MAX; ++ss)
                    v[ss] = ss < S ? __hip_atomic_load(a.ks_part + ((size_t)ss * n_groups + g) * 256 + row * 16 + col,
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                   : 0.f;
#pragma unroll
                for (int ss = 0; ss < KSPLIT_MAX; ++ss) sum += v[ss];  // slice order; absent slices add an exact zero
            }
            my_tile[row * 17 + col] = sum;
        }
        __syncthreads();
        if (mine) {
            if constexpr (PRE) epilogue_tile_pre<EPI>(a, my_tile, 17, s_scale, R, g, Ntot, tl, pre);
            else epilogue_tile<EPI, 16, 256>(a, my_tile, 17, s_scale, R, g, Ntot, tl);
        }
        __syncthreads();
    }
}

// ---- 8-bit weights, any shape ---------------------------------------------------------------------------
// One workgroup per 16-row group of W, its NW waves split the group's 64-k tiles in contiguous slices (the shapes
// the persistent kernel does not take: K = 14336, more than 16 rows, K not a multiple of 1024).  Per burst a wave
// issues U tile loads, then per tile and half gathers the x fragments of every row block, turns the half tile into
// bf16 and multiplies.  Reduction, row scales and epilogues as in gemv_mfma_k; the column scales of the weights are
// multiplied into the reduced tile.
template <int EPI, int MB, int NW>
__global__ __launch_bounds__(NW * 64) void gemv_q8_k(const GemvArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int NT = NW * 64;
    constexpr int FR = MB * 256;
    constexpr int TS = 17;
    constexpr int U = MB == 1 ? 8 : (MB == 2 ? 4 : (MB == 4 ? 2 : 1));  // tile loads in flight per wave
    static_assert(NW * MB <= 32, "partial tiles must fit 32 KiB of LDS");
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: see above
    int Ntot = a.n0;
    if (EPI == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (EPI == EPI_SWIGLU) Ntot = 2 * a.n0;
    const int g = blockIdx.x;
    const int K = a.K, KT = K >> 6;
    const int KTw = (KT + NW - 1) / NW;
    const int kt_begin = min(wave * KTw, KT), kt_end = min(kt_begin + KTw, KT);
    const int R = a.R;

    __shared__ float part[NW * FR];
    __shared__ float tile[MB * 16 * TS];
    __shared__ float s_scale[MB * 16];

    RowScales<NT> rs;
    rs.begin(a, R);

    const u32x4_t *bp = reinterpret_cast<const u32x4_t *>(a.w0) + ((size_t)g * KT + kt_begin) * 64 + lane;
    const bool has_lo = a.xb_lo != 0;
    const bool fold = has_lo && MB == 1 && R <= 8;  // hi rows in 0..7, lo rows in 8..15 of one fragment
    const bool two_terms = has_lo && !fold;
    const uint16_t *ap[MB];
    bool row_ok[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        int r = mb * 16 + (lane & 15);
        size_t off = 0;
        if (fold && r >= 8) { r -= 8; off = (size_t)a.xb_lo; }
        row_ok[mb] = r < R;
        const size_t xr = (size_t)(min(r, R - 1) * a.x_mul + a.x_add);
        ap[mb] = a.xb + off + xr * K + (size_t)kt_begin * 64 + (lane >> 4) * 16;
    }
    f32x4_t acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    if constexpr (MB == 1) {
        // one row block: two half-size batches of tiles in registers, the next requested before this one's matrix
        // instructions, after the x fragments of the whole batch (a younger load would make waiting for them wait
        // for the weight tiles too)
        constexpr int UP = U / 2;
        u32x4_t bwA[UP], bwB[UP];
        auto load_w = [&](u32x4_t(&bw)[UP], int kt) {
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (kt + u < kt_end) bw[u] = __builtin_nontemporal_load(bp + 64 * (kt - kt_begin + u));
        };
        auto batch = [&](const u32x4_t(&bw)[UP], u32x4_t(&next)[UP], int kt) {
            u32x4_t xh[UP][2], xl[UP][2];
#pragma unroll
            for (int u = 0; u < UP; ++u)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    xh[u][h] = u32x4_t{0u, 0u, 0u, 0u};
                    xl[u][h] = u32x4_t{0u, 0u, 0u, 0u};
                    if (kt + u < kt_end && row_ok[0]) {
                        const uint16_t *xp = ap[0] + (size_t)(kt - kt_begin + u) * 64 + h * 8;
                        xh[u][h] = *reinterpret_cast<const u32x4_t *>(xp);
                        if (two_terms) xl[u][h] = *reinterpret_cast<const u32x4_t *>(xp + a.xb_lo);
                    }
                }
            load_w(next, kt + UP);
#pragma unroll
            for (int u = 0; u < UP; ++u) {
                if (kt + u < kt_end) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const u32x4_t wb = q8_half_to_bf16(h == 0 ? q8_u32x2_t{bw[u].x, bw[u].y} : q8_u32x2_t{bw[u].z, bw[u].w});
                        acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xh[u][h]),
                                                                         __builtin_bit_cast(bf16x8_t, wb), acc[0], 0, 0, 0);
                        if (two_terms)
                            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xl[u][h]),
                                                                             __builtin_bit_cast(bf16x8_t, wb), acc[0], 0, 0, 0);
                    }
                }
            }
        };
        load_w(bwA, kt_begin);
        for (int kt = kt_begin; kt < kt_end; kt += 2 * UP) {
            batch(bwA, bwB, kt);
            if (kt + UP < kt_end) batch(bwB, bwA, kt + UP);
        }
    } else
    for (int kt = kt_begin; kt < kt_end; kt += U) {
        u32x4_t bw[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (kt + u < kt_end) bw[u] = __builtin_nontemporal_load(bp + 64 * u);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kt + u < kt_end) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    u32x4_t xh[MB], xl[MB];
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        xh[mb] = u32x4_t{0u, 0u, 0u, 0u};
                        xl[mb] = u32x4_t{0u, 0u, 0u, 0u};
                        if (row_ok[mb]) {
                            xh[mb] = *reinterpret_cast<const u32x4_t *>(ap[mb] + u * 64 + h * 8);
                            if (two_terms) xl[mb] = *reinterpret_cast<const u32x4_t *>(ap[mb] + a.xb_lo + u * 64 + h * 8);
                        }
                    }
                    const u32x4_t wb = q8_half_to_bf16(h == 0 ? q8_u32x2_t{bw[u].x, bw[u].y} : q8_u32x2_t{bw[u].z, bw[u].w});
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xh[mb]),
                                                                          __builtin_bit_cast(bf16x8_t, wb), acc[mb], 0, 0, 0);
                        if (two_terms)
                            acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xl[mb]),
                                                                              __builtin_bit_cast(bf16x8_t, wb), acc[mb], 0, 0, 0);
                    }
                }
            }
        }
        bp += 64 * U;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) ap[mb] += 64 * U;
    }

#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave * FR + ((mb * 4 + v) << 6) + lane] = acc[mb][v];
    __syncthreads();
    for (int idx = threadIdx.x; idx < FR; idx += NT) {
        float s = part[idx];
#pragma unroll
        for (int w = 1; w < NW; ++w) s += part[w * FR + idx];
        const int l = idx & 63, v = (idx >> 6) & 3, mb = idx >> 8;
        if (fold) {
            if (l >= 32) continue;
            float s2 = part[idx + 32];
#pragma unroll
            for (int w = 1; w < NW; ++w) s2 += part[w * FR + idx + 32];
            s += s2;
        }
        tile[(mb * 16 + (l >> 4) * 4 + v) * TS + (l & 15)] = s * a.wscale[(size_t)g * 16 + (l & 15)];
    }
    rs.finish(a, s_scale, R);  // ends with a barrier
    epilogue_tile<EPI, 16, NT>(a, tile, TS, s_scale, R, g, Ntot, threadIdx.x);
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

int gemv_mfma_groups_per_wg(int epi, int Ntot, int K, int R, int forced, bool q8) {
    (void)epi;
    if (q8) return 1;
    if (forced == 0 && gemv_mfma_resident_x(K, R, q8)) return 1;  // the engine's activations carry two terms
    const int MB = R <= 16 ? 1 : (R <= 32 ? 2 : (R <= 64 ? 4 : 8));
    return pick_cfg(Ntot / 16, K / 32, MB, forced).ng;
}

// Events of an optional timed launch: recorded by the dispatch itself (start and end of the kernel,
// nothing of the launch path in between).
struct LaunchEvents { hipEvent_t start, stop; };

// Compute units of the current device, read once per device (the persistent kernel launches one workgroup per unit).
static int compute_units() {
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

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

// The persistent kernel serves one 16-row block of x whose fragments fit the registers of a 16-wave workgroup:
// K <= 512 KTW with KTW x (1 or 2 fragments) <= 20, KTW in {2, 3, 4, 6, 8, 10, 16} (the 768-, 1536-, 2048-, 3072-,
// 4096-, 5120- and 8192-wide projections of the model shapes at hand; K = 768 fills its second round half).
static int persist_terms(const GemvArgs &a) { return (a.xb_lo != 0 && a.R > 8) ? 2 : 1; }
static int persist_ktw(const GemvArgs &a) { return (a.K / 32 + PW - 1) / PW; }
static bool persist_fits(const GemvArgs &a) {
    if (a.R > 16 || a.K % 32) return false;
    const int ktw = persist_ktw(a);
    const bool ragged = a.K % 512 != 0;
    if (a.wscale != nullptr) {  // 8-bit tiles span 64 k: 16 waves x 64, whole rounds only
        if (a.K % 1024 || (ktw != 4 && ktw != 8 && ktw != 16)) return false;
    } else {
        if (ktw != 2 && ktw != 3 && ktw != 4 && ktw != 6 && ktw != 8 && ktw != 10 && ktw != 16) return false;
        if (ragged && ktw != 2) return false;
    }
    return ktw * persist_terms(a) <= 20;
}

template <int EPI, int KTW, int TERMS, int WQ, int RAG = 0>
static hipError_t launch_persist_one(const GemvArgs &a, int n_groups, LaunchEvents ev, hipStream_t s) {
    const int cus = compute_units();
    const int G = n_groups < cus ? n_groups : cus;  // one workgroup per compute unit
    if (ev.start != nullptr)
        hipExtLaunchKernelGGL((gemv_persist_k<EPI, KTW, TERMS, WQ, RAG>), dim3(G), dim3(PW * 64), 0, s, ev.start, ev.stop, 0, a);
    else
        hipLaunchKernelGGL((gemv_persist_k<EPI, KTW, TERMS, WQ, RAG>), dim3(G), dim3(PW * 64), 0, s, a);
    return hipGetLastError();
}

template <int EPI, int WQ>
static hipError_t launch_persist(const GemvArgs &a, int n_groups, LaunchEvents ev, hipStream_t s) {
    const int ktw = persist_ktw(a);
    const bool two = persist_terms(a) == 2;
    if constexpr (WQ == 0) {
        if (a.K % 512) return two ? launch_persist_one<EPI, 2, 2, 0, 1>(a, n_groups, ev, s) : launch_persist_one<EPI, 2, 1, 0, 1>(a, n_groups, ev, s);
        switch (ktw) {
            case 2: return two ? launch_persist_one<EPI, 2, 2, 0>(a, n_groups, ev, s) : launch_persist_one<EPI, 2, 1, 0>(a, n_groups, ev, s);
            case 3: return two ? launch_persist_one<EPI, 3, 2, 0>(a, n_groups, ev, s) : launch_persist_one<EPI, 3, 1, 0>(a, n_groups, ev, s);
            case 6: return two ? launch_persist_one<EPI, 6, 2, 0>(a, n_groups, ev, s) : launch_persist_one<EPI, 6, 1, 0>(a, n_groups, ev, s);
            case 10: return two ? launch_persist_one<EPI, 10, 2, 0>(a, n_groups, ev, s) : launch_persist_one<EPI, 10, 1, 0>(a, n_groups, ev, s);
            default: break;
        }
    }
    if (two) {
        if (ktw == 4) return launch_persist_one<EPI, 4, 2, WQ>(a, n_groups, ev, s);
        return launch_persist_one<EPI, 8, 2, WQ>(a, n_groups, ev, s);
    }
    if (ktw == 4) return launch_persist_one<EPI, 4, 1, WQ>(a, n_groups, ev, s);
    if (ktw == 8) return launch_persist_one<EPI, 8, 1, WQ>(a, n_groups, ev, s);
    return launch_persist_one<EPI, 16, 1, WQ>(a, n_groups, ev, s);
}

// The persistent kernel for 17 to 64 rows: the x fragments of MB row blocks, KTW k-tiles per wave and `terms` bf16
// terms fit 16 registers-of-four.
static bool persist_mb_shape(int K, int R, int terms, bool q8) {
    if (q8 || R <= 16 || R > 64 || K % 32) return false;
    const int MB = R <= 32 ? 2 : (R <= 48 ? 3 : 4);
    const int ktw = (K / 32 + PW - 1) / PW;
    if (K % 512 && ktw > 2) return false;   // a short last round is compiled for K < 1024 only
    return (ktw == 1 || ktw == 2 || ktw == 4) && MB * ktw * terms <= 16;
}

bool gemv_mfma_resident_x(int K, int R, bool q8) {
    static const bool off = std::getenv("SPEC_NO_PERSIST_MB") != nullptr;  // measurement aid
    return !off && persist_mb_shape(K, R, 2, q8);
}

template <int EPI, int KTW, int MB, int TERMS>
static hipError_t launch_persist_mb_one(const GemvArgs &a, int n_groups, LaunchEvents ev, hipStream_t s) {
    if constexpr (MB * KTW * TERMS <= 16) {
        const int cus = compute_units();
        const int G = n_groups < cus ? n_groups : cus;
        auto go = [&](auto kern) {
            if (ev.start != nullptr) hipExtLaunchKernelGGL(kern, dim3(G), dim3(PW * 64), 0, s, ev.start, ev.stop, 0, a);
            else hipLaunchKernelGGL(kern, dim3(G), dim3(PW * 64), 0, s, a);
            return hipGetLastError();
        };
        if constexpr (KTW <= 2) {
            if (a.K % 512) return go(gemv_persist_mb_k<EPI, KTW, MB, TERMS, 1>);
        }
        return go(gemv_persist_mb_k<EPI, KTW, MB, TERMS, 0>);
    } else {
        return hipErrorInvalidValue;
    }
}

template <int EPI, int MB>
static hipError_t launch_persist_mb(const GemvArgs &a, int n_groups, LaunchEvents ev, hipStream_t s) {
    const int ktw = (a.K / 32 + PW - 1) / PW;
    const bool two = a.xb_lo != 0;
    switch (ktw) {
        case 1: return two ? launch_persist_mb_one<EPI, 1, MB, 2>(a, n_groups, ev, s) : launch_persist_mb_one<EPI, 1, MB, 1>(a, n_groups, ev, s);
        case 2: return two ? launch_persist_mb_one<EPI, 2, MB, 2>(a, n_groups, ev, s) : launch_persist_mb_one<EPI, 2, MB, 1>(a, n_groups, ev, s);
        case 4: return two ? launch_persist_mb_one<EPI, 4, MB, 2>(a, n_groups, ev, s) : launch_persist_mb_one<EPI, 4, MB, 1>(a, n_groups, ev, s);
    }
    return hipErrorInvalidValue;
}

// Slices of K for the kernel that shares K out over workgroups (0: that kernel does not serve the shape).
static int ksplit_slices(const GemvArgs &a, int epi, int n_groups) {
    static const bool off = std::getenv("SPEC_NO_KSPLIT") != nullptr;  // measurement aid: route as if the kernel were absent
    if (off || a.ks_part == nullptr || a.ks_ticket == nullptr || a.wscale != nullptr) return 0;
    if (a.R > 16 || a.K % 32) return 0;
    const int KT = a.K / 32, terms = persist_terms(a), cus = compute_units();
    const bool plain = epi == EPI_PLAIN || epi == EPI_RESID;
    // Where the persistent kernel serves the shape it stays, unless it leaves half the compute units idle on a long
    // K (the 1B-shaped down projection: 128 groups of K = 8192), or both bf16 terms of x take 80 registers there
    // (K = 5120 at 9 to 16 rows: two slices of five k-tiles per wave leave room for full load bursts; 13B-shaped pass
    // of 16 rows 7.36 -> 6.54 ms).  Measured and not taken: two slices for the K = 4096 projections of the 8B-shaped
    // target (QKV 12.3 -> 13.6 us, gate/up 39.0 -> 43.6, LM head 167 -> 193: the persistent kernel is the faster one
    // wherever its fragments fit).  Measured
    // and not taken: sharing K out where the persistent kernel's last round of groups is mostly empty (13B-shaped
    // output projection, 320 groups on 256 units) - the counter and the finish cost what the even rounds save.
    if (persist_fits(a)) {
        const int ktw = persist_ktw(a);
        if (ktw * terms >= 20 && KT % 2 == 0 && ((KT / 2 + PW - 1) / PW) == 5 && KT / 2 == 5 * PW) return 2;
        if (!(plain && 2 * n_groups <= cus && KT >= 256)) return 0;
    }
    if (!plain) return 0;  // the long-K shapes are down projections
    for (int S = 2; S <= KSPLIT_MAX; S *= 2) {
        if (KT % S || n_groups * S < cus / 2) continue;
        const int ktw = (KT / S + PW - 1) / PW;
        if (ktw >= 6 && ktw <= 8 && ktw * terms <= 16) return S;
    }
    return 0;
}

template <int EPI, int KTW, int TERMS>
static hipError_t launch_ksplit_one(const GemvArgs &a, int S, int J, bool ragged, LaunchEvents ev, hipStream_t s) {
    // instances: five k-tiles per wave with both terms for every epilogue; six to eight for the down projections
    if constexpr ((KTW == 5 && TERMS == 2) || (KTW >= 6 && (EPI == EPI_PLAIN || EPI == EPI_RESID))) {
        auto go = [&](auto kern) {
            if (ev.start != nullptr) hipExtLaunchKernelGGL(kern, dim3(S * J), dim3(PW * 64), 0, s, ev.start, ev.stop, 0, a, S);
            else hipLaunchKernelGGL(kern, dim3(S * J), dim3(PW * 64), 0, s, a, S);
            return hipGetLastError();
        };
        if constexpr (KTW <= 5) return ragged ? hipErrorInvalidValue : go(gemv_ksplit_k<EPI, KTW, TERMS, 0>);
        else return ragged ? go(gemv_ksplit_k<EPI, KTW, TERMS, 1>) : go(gemv_ksplit_k<EPI, KTW, TERMS, 0>);
    } else {
        return hipErrorInvalidValue;
    }
}

template <int EPI>
static hipError_t launch_ksplit(const GemvArgs &a, int S, int n_groups, LaunchEvents ev, hipStream_t s) {
    const int cus = compute_units();
    int J = cus / S;
    if (J > n_groups) J = n_groups;
    if (J > KSPLIT_TICKETS) J = KSPLIT_TICKETS;
    const int KTs = a.K / 32 / S, ktw = (KTs + PW - 1) / PW;
    const bool ragged = KTs % PW != 0, two = persist_terms(a) == 2;
    switch (ktw) {
        case 5: return two ? launch_ksplit_one<EPI, 5, 2>(a, S, J, ragged, ev, s) : hipErrorInvalidValue;
        case 6: return two ? launch_ksplit_one<EPI, 6, 2>(a, S, J, ragged, ev, s) : launch_ksplit_one<EPI, 6, 1>(a, S, J, ragged, ev, s);
        case 7: return two ? launch_ksplit_one<EPI, 7, 2>(a, S, J, ragged, ev, s) : launch_ksplit_one<EPI, 7, 1>(a, S, J, ragged, ev, s);
        case 8: return two ? launch_ksplit_one<EPI, 8, 2>(a, S, J, ragged, ev, s) : launch_ksplit_one<EPI, 8, 1>(a, S, J, ragged, ev, s);
    }
    return hipErrorInvalidValue;
}

template <int EPI>
static hipError_t launch_cfg(const GemvArgs &a, int Ntot, int forced, LaunchEvents ev, hipStream_t s) {
    const int MB = a.R <= 16 ? 1 : (a.R <= 32 ? 2 : (a.R <= 64 ? 4 : 8));
    const int n_groups = Ntot / 16;
    if (a.wscale != nullptr) {
        if (a.K % 64) return hipErrorInvalidValue;
        if (forced == 0 && persist_fits(a)) return launch_persist<EPI, 1>(a, n_groups, ev, s);
        auto go = [&](auto kern, int nw) {
            if (ev.start != nullptr) hipExtLaunchKernelGGL(kern, dim3(n_groups), dim3(nw * 64), 0, s, ev.start, ev.stop, 0, a);
            else hipLaunchKernelGGL(kern, dim3(n_groups), dim3(nw * 64), 0, s, a);
            return hipGetLastError();
        };
        switch (MB) {
            case 1: return go(gemv_q8_k<EPI, 1, 8>, 8);
            case 2: return go(gemv_q8_k<EPI, 2, 8>, 8);
            case 4: return go(gemv_q8_k<EPI, 4, 8>, 8);
            default: return go(gemv_q8_k<EPI, 8, 4>, 4);
        }
    }
    if (forced == 0) {
        const int S = ksplit_slices(a, EPI, n_groups);
        if (S > 0) return launch_ksplit<EPI>(a, S, n_groups, ev, s);
        static const bool mb_off = std::getenv("SPEC_NO_PERSIST_MB") != nullptr;
        if (!mb_off && persist_mb_shape(a.K, a.R, a.xb_lo != 0 ? 2 : 1, false)) {
            if (a.R <= 32) return launch_persist_mb<EPI, 2>(a, n_groups, ev, s);
            if (a.R <= 48) return launch_persist_mb<EPI, 3>(a, n_groups, ev, s);
            return launch_persist_mb<EPI, 4>(a, n_groups, ev, s);
        }
    }
    if (forced == 0 && persist_fits(a)) return launch_persist<EPI, 0>(a, n_groups, ev, s);
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
