// Attention of the rows of one forward pass against the paged KV cache, split over KV chunks
// (partial softmax per chunk, merged by a combine kernel).  The rows of a sequence are the
// gamma+1 verification rows of the target, or the 1-2 decode rows of the draft; row i may see
// cache positions <= its own position (causal inside the rows).
//
// attn_simple_k is the plain version: any head size and cache type, fp32 arithmetic, one
// workgroup per (chunk, query head, sequence).  It serves fp32 models.
#include <cstdlib>

#include "common.hpp"
#include "kv.hpp"
#include "params.hpp"

namespace sd {

constexpr int ATT_CT = 64;        // KV positions per chunk
constexpr int ATT_RPS_MAX = 128;  // rows per sequence the simple kernel can hold

__global__ __launch_bounds__(256) void attn_simple_k(const AttnArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int hd = a.kv.hd;
    const int kvh = h / (a.nq / a.kv.n_kv);
    const int r_first = b * a.rps;
    const int t0 = c * ATT_CT;
    const int last_pos = a.row_pos[r_first + a.rps - 1];
    if (t0 > last_pos) return;  // nothing of this chunk is visible to any row

    __shared__ float S[ATT_RPS_MAX][ATT_CT + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // scores
    for (int idx = threadIdx.x; idx < a.rps * ATT_CT; idx += 256) {
        const int i = idx / ATT_CT, t = idx % ATT_CT;
        const int r = r_first + i;
        const int pos = t0 + t;
        float s = -INFINITY;
        if (pos <= a.row_pos[r]) {
            const float *q = a.q + ((size_t)r * a.nq + h) * hd;
            const size_t kb = kv_head_base(a.kv, kv_page(a.kv, b, pos), kvh);
            const int tp = pos & (a.kv.page_tokens - 1);
            float acc = 0.f;
            for (int e = 0; e < hd; ++e) acc = fmaf(q[e], kv_load(a.kv.k, a.kv_dtype, kb + kv_in_k(a.kv, tp, e)), acc);
            s = acc * a.scale;
        }
        S[i][t] = s;
    }
    __syncthreads();
    // chunk-local softmax statistics: one wave per row, one lane per position
    for (int i = wave; i < a.rps; i += 4) {
        const float s = S[i][lane];
        const float m = wave_max(s);
        const float p = m == -INFINITY ? 0.f : __expf(s - m);
        const float l = wave_sum(p);
        S[i][lane] = p;
        if (lane == 0) {
            const size_t pi = ((size_t)(r_first + i) * a.nq + h) * a.n_chunks + c;
            a.part_m[pi] = m;
            a.part_l[pi] = l;
        }
    }
    __syncthreads();
    // weighted values
    for (int idx = threadIdx.x; idx < a.rps * hd; idx += 256) {
        const int i = idx / hd, e = idx % hd;
        float acc = 0.f;
        const int tmax = min(ATT_CT, last_pos - t0 + 1);
        for (int t = 0; t < tmax; ++t) {
            const float p = S[i][t];
            if (p != 0.f) acc = fmaf(p, kv_load(a.kv.v, a.kv_dtype, kv_index_v(a.kv, b, t0 + t, kvh, e)), acc);
        }
        a.part_o[(((size_t)(r_first + i) * a.nq + h) * a.n_chunks + c) * hd + e] = acc;
    }
}

// Merge the chunk partials of one (row, head): o = sum_c exp(m_c - M) o_c / sum_c exp(m_c - M) l_c.
__global__ __launch_bounds__(128) void attn_combine_k(const AttnArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    const int r = blockIdx.x, h = blockIdx.y;
    const int hd = a.kv.hd;
    const int nc = a.row_pos[r] / ATT_CT + 1;  // chunks that hold a visible position
    const size_t pb = ((size_t)r * a.nq + h) * a.n_chunks;
    float M = -INFINITY;
    for (int c = 0; c < nc; ++c) M = fmaxf(M, a.part_m[pb + c]);
    float L = 0.f;
    for (int c = 0; c < nc; ++c) L += a.part_l[pb + c] * __expf(a.part_m[pb + c] - M);
    const float inv = 1.f / L;
    for (int e = threadIdx.x; e < hd; e += 128) {
        float acc = 0.f;
        for (int c = 0; c < nc; ++c) acc += __expf(a.part_m[pb + c] - M) * a.part_o[(pb + c) * hd + e];
        const float v = acc * inv;
        const size_t o = ((size_t)r * a.nq + h) * hd + e;
        a.o[o] = v;
        a.ob[o] = f32_to_bf16(v);
    }
}

// ---- matrix-core version for 16-bit caches --------------------------------------------------------
// One workgroup per (chunk of 64 * SPW positions, kv head, sequence); wave w owns the 16-position slabs
// w, w + 4, ... of the chunk.  A wave first issues every load of its slabs (K and V fragments
// - kv.hpp - straight into the operand layouts; positions past the last visible one are clamped, so the
// loads and the matrix instructions need no branch), then per 16-query tile forms S^T = K Q^T with
// v_mfma_f32_16x16x32_bf16, takes the softmax over its slabs, and multiplies by V with
// v_mfma_f32_16x16x16_bf16: the S^T result registers already are the A operand (query = lane % 16, four
// positions per lane).  The four wave partials are merged through LDS into one (max, sum, vector)
// partial per chunk, and attn_mfma_merge_k merges the chunk partials into the attention output (a
// kernel boundary is the cheapest way to order the partials across the chip's eight L2 caches).  A
// sequence that fits one chunk skips the partials.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint64_t pack_f32x2(float lo, float hi) {
    return (uint64_t)__float_as_uint(lo) | ((uint64_t)__float_as_uint(hi) << 32);
}
__device__ __forceinline__ float f32_lo(uint64_t u) { return __uint_as_float((uint32_t)u); }
__device__ __forceinline__ float f32_hi(uint64_t u) { return __uint_as_float((uint32_t)(u >> 32)); }

constexpr int ATT_SPW_MAX = 8;   // slabs per wave -> chunks of up to 512 positions
constexpr int ATT_TILES_PER_WG = 8;  // 16-query tiles a workgroup works through (decode and verification: all of them)

// AHEAD: the row-dependent loads (a sequence's last position, the queries of the tile after this one) are held a
// step ahead in registers - shorter dependent chains for the few workgroups of a single sequence, but 30-40 more
// registers, which cost a workgroup per compute unit when a batch launches thousands.
// FUSE: the chunk partials of a (sequence, kv head) are merged by whichever of its workgroups finishes last, instead
// of by attn_mfma_merge_k: the partials are written with agent-scope stores (past the per-XCD L2 caches), every
// workgroup then takes a ticket from the pair's arrival counter, and the one that draws the last ticket reads all
// partials back with agent-scope loads and merges them with the arithmetic of the merge kernel, in chunk order.
// For launches of few workgroups (one or a few sequences), where a second launch costs more than the tail does.
template <int HD, int SPW, bool AHEAD, bool FUSE = false>
__global__ __launch_bounds__(256) void attn_mfma_k(const AttnArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int ES = HD / 32;  // k-steps of the score product
    constexpr int ET = HD / 16;  // 16-channel tiles of the output
    constexpr int CT = 64 * SPW;
    // grid.z = sequences x query splits: with many rows per sequence (prompt ingestion) the 16-query tiles of a
    // sequence are shared out over several workgroups, each of which loads the chunk for itself
    const int QS = gridDim.z / a.batch;
    const int c = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z / QS, qs = blockIdx.z % QS;
    // wave index and last position are scalars, so that branches on them are scalar branches
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int G = a.nq / a.kv.n_kv;
    // rows of this sequence: a.rps each, or its own count when the sequences of a verification pass differ
    const int r_first = a.row_off != nullptr ? a.row_off[b] : b * a.rps;
    const int rps = a.row_off != nullptr ? a.row_off[b + 1] - r_first : a.rps;
    if (rps <= 0) return;  // a sequence without rows in this pass (draft passes over the sequences still drafting)
    const int QN = G * rps;
    const int t0 = c * CT;
    const bf16_t *kp = reinterpret_cast<const bf16_t *>(a.kv.k);
    const bf16_t *vp = reinterpret_cast<const bf16_t *>(a.kv.v);

    __shared__ __attribute__((aligned(16))) float sO[4][16][HD + 4];  // rows 16-byte aligned, 4 g apart on different banks
    __shared__ float sM[4][16], sL[4][16];

    // K fragment: position tw + l16, channels 32 s + 8 g .. + 8; V fragment: channel 16 et + l16, positions
    // tw + 4 g .. + 4 (eight contiguous bytes in either arrangement of the page).  Positions are clamped to the cache capacity only, not to
    // the sequence length: the loads then depend on nothing but the block table and start at once; whatever finite
    // values lie beyond the last visible position meet a zero probability.
    const int cap = a.kv.pages_per_seq * a.kv.page_tokens;
    // What depends on the rows alone goes out first: the sequence's last position and the first tile's queries are
    // older loads than the K / V fragments below, so waiting for them does not wait for the cache, and they are in
    // flight while the block table is looked up.
    const bool has_qlo = a.qb_lo != 0;
    const int QT = (QN + 15) / 16, TPW = (QT + QS - 1) / QS;
    const int last_pos_l = a.row_pos[r_first + rps - 1];
    struct QTile { int qpos; u32x4_t qf[ES], ql[ES]; };
    auto load_q = [&](int qt, QTile &q) {
        // query handled by this lane in the score product (column l16 of S^T); q enters as hi + lo bf16 terms
        const int qi = min(qt * 16 + l16, QN - 1);
        const int gq = qi / rps, i = qi % rps;
        const int r = r_first + i, h = kvh * G + gq;
        q.qpos = a.row_pos[r];
        const bf16_t *qp = a.qb + ((size_t)r * a.nq + h) * HD + 8 * g;
#pragma unroll
        for (int s = 0; s < ES; ++s) {
            q.qf[s] = *reinterpret_cast<const u32x4_t *>(qp + 32 * s);
            q.ql[s] = has_qlo ? *reinterpret_cast<const u32x4_t *>(qp + a.qb_lo + 32 * s) : u32x4_t{0u, 0u, 0u, 0u};
        }
    };
    QTile qn;
    if constexpr (AHEAD) load_q(qs * TPW, qn);
    u32x4_t kf[SPW][ES];
    u32x2_t vf[SPW][ET];
    const int k_step = kv_step_k(a.kv), v_step = kv_step_v(a.kv);
#pragma unroll
    for (int sl = 0; sl < SPW; ++sl) {
        const int tw = t0 + 16 * (wave + 4 * sl);
        const int pk = min(tw + l16, cap - 1);
        const size_t kb = kv_index_k(a.kv, b, pk, kvh, 8 * g);
#pragma unroll
        for (int s = 0; s < ES; ++s) kf[sl][s] = *reinterpret_cast<const u32x4_t *>(kp + kb + (size_t)s * k_step);
        const int pv = min(tw + 4 * g, cap - 4);
        const size_t vb = kv_index_v(a.kv, b, pv, kvh, l16);
#pragma unroll
        for (int et = 0; et < ET; ++et)
            vf[sl][et] = *reinterpret_cast<const u32x2_t *>(vp + vb + (size_t)et * v_step);
    }
    const int last_pos = __builtin_amdgcn_readfirstlane(last_pos_l);
    if (t0 > last_pos) return;
    const int n_live = last_pos / CT + 1;

    const int qt_end = min(QT, (qs + 1) * TPW);
    for (int qt = qs * TPW; qt < qt_end; ++qt) {
        // this tile's queries were requested a tile ago and the next tile's go out now, or every tile loads its own
        if constexpr (!AHEAD) load_q(qt, qn);
        const QTile qc = qn;
        if (AHEAD && qt + 1 < qt_end) load_q(qt + 1, qn);
        const int qpos = qc.qpos;
        // a tile none of whose queries sees this chunk leaves no partial: the merge never reads one there
        if (t0 > __builtin_amdgcn_readfirstlane(wave_max(qpos))) continue;
        const u32x4_t(&qf)[ES] = qc.qf;
        const u32x4_t(&ql)[ES] = qc.ql;
        // scores of every slab of this wave; S[sl][v] = (position tw + 4 g + v, query l16)
        f32x4_t S[SPW];
        float m = -INFINITY;
#pragma unroll
        for (int sl = 0; sl < SPW; ++sl) {
            const int tw = t0 + 16 * (wave + 4 * sl);
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < ES; ++s) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[sl][s]),
                                                              __builtin_bit_cast(bf16x8_t, qf[s]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[sl][s]),
                                                              __builtin_bit_cast(bf16x8_t, ql[s]), acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool vis = (tw + 4 * g + v) <= qpos;
                S[sl][v] = vis ? acc[v] * a.scale : -INFINITY;
                m = fmaxf(m, S[sl][v]);
            }
        }
        m = fmaxf(m, __shfl_xor(m, 16, WAVE));
        m = fmaxf(m, __shfl_xor(m, 32, WAVE));
        // probabilities and the weighted values
        float l = 0.f;
        f32x4_t O[ET];
#pragma unroll
        for (int et = 0; et < ET; ++et) O[et] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sl = 0; sl < SPW; ++sl) {
            float p[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                p[v] = m == -INFINITY ? 0.f : __expf(S[sl][v] - m);
                l += p[v];
            }
            // probabilities as hi + lo bf16 terms as well
            u32x2_t pw, pl;
            pw.x = pack_bf16x2(p[0], p[1]);
            pw.y = pack_bf16x2(p[2], p[3]);
            pl.x = pack_bf16x2(p[0] - bf16_lo(pw.x), p[1] - bf16_hi(pw.x));
            pl.y = pack_bf16x2(p[2] - bf16_lo(pw.y), p[3] - bf16_hi(pw.y));
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                O[et] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, pw),
                                                                  __builtin_bit_cast(s16x4_t, vf[sl][et]), O[et], 0, 0, 0);
                O[et] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, pl),
                                                                  __builtin_bit_cast(s16x4_t, vf[sl][et]), O[et], 0, 0, 0);
            }
        }
        l += __shfl_xor(l, 16, WAVE);
        l += __shfl_xor(l, 32, WAVE);
        if (g == 0) { sM[wave][l16] = m; sL[wave][l16] = l; }
        // result register v of lane (channel l16, g) is query 4 g + v
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int v = 0; v < 4; ++v) sO[wave][4 * g + v][16 * et + l16] = O[et][v];
        __syncthreads();
        // merge the four wave partials: thread -> (query, HD / 16 consecutive channels), so that the weights of a
        // query's four partials are formed once per thread and the channels move as vectors
        {
            constexpr int EPT = HD / 16;
            const int q = threadIdx.x >> 4, e0 = (threadIdx.x & 15) * EPT;
            const int qj = qt * 16 + q;
            if (qj < QN) {
                const float M = fmaxf(fmaxf(sM[0][q], sM[1][q]), fmaxf(sM[2][q], sM[3][q]));
                float f[4], L = 0.f, acc[EPT];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    f[w] = sM[w][q] == -INFINITY ? 0.f : __expf(sM[w][q] - M);
                    L += f[w] * sL[w][q];
                }
#pragma unroll
                for (int k = 0; k < EPT; ++k) acc[k] = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w)
#pragma unroll
                    for (int k = 0; k < EPT; ++k) acc[k] += f[w] * sO[w][q][e0 + k];
                const int rr = r_first + qj % rps, hh = kvh * G + qj / rps;
                if (n_live == 1) {
                    const size_t o = ((size_t)rr * a.nq + hh) * HD + e0;
#pragma unroll
                    for (int k = 0; k < EPT; ++k) {
                        const float v = acc[k] / L;
                        a.o[o + k] = v;
                        store_split_bf16(a.ob, o + k, a.ob_lo, v);
                    }
                } else {
                    const size_t pi = ((size_t)rr * a.nq + hh) * a.n_chunks + c;
                    float *po = a.part_o + pi * HD + e0;
                    if constexpr (FUSE) {
#pragma unroll
                        for (int k = 0; k < EPT; k += 2)
                            __hip_atomic_store(reinterpret_cast<uint64_t *>(po + k), pack_f32x2(acc[k], acc[k + 1]),
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (e0 == 0) {
                            __hip_atomic_store(a.part_m + pi, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            __hip_atomic_store(a.part_l + pi, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    } else if constexpr (EPT % 4 == 0) {
#pragma unroll
                        for (int k = 0; k < EPT; k += 4)
                            *reinterpret_cast<f32x4_t *>(po + k) = f32x4_t{acc[k], acc[k + 1], acc[k + 2], acc[k + 3]};
                    } else {
#pragma unroll
                        for (int k = 0; k < EPT; ++k) po[k] = acc[k];
                    }
                    if (!FUSE && e0 == 0) { a.part_m[pi] = M; a.part_l[pi] = L; }
                }
            }
        }
        __syncthreads();
    }
    if constexpr (FUSE) {
        if (n_live == 1) return;  // the output was written above
        __shared__ int s_last;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's partial stores have been acknowledged
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t *tk = a.ticket + (size_t)b * a.kv.n_kv + kvh;
            const uint32_t old = __hip_atomic_fetch_add(tk, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == (uint32_t)(n_live - 1);
            if (s_last) __hip_atomic_store(tk, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next launch
        }
        __syncthreads();
        if (!s_last) return;
        constexpr int EPT = HD / 16, NCB = 16;  // host: at most 16 chunks
        const int q = threadIdx.x >> 4, e0 = (threadIdx.x & 15) * EPT;
        for (int qt = qs * TPW; qt < qt_end; ++qt) {
            const int qj = qt * 16 + q;
            if (qj >= QN) continue;
            const int rr = r_first + qj % rps, hh = kvh * G + qj / rps;
            const size_t pb = ((size_t)rr * a.nq + hh) * a.n_chunks;
            float pm[NCB], pl[NCB];
            uint64_t po[NCB][EPT / 2];
#pragma unroll
            for (int cc = 0; cc < NCB; ++cc) {
                pm[cc] = -INFINITY; pl[cc] = 0.f;
#pragma unroll
                for (int k = 0; k < EPT / 2; ++k) po[cc][k] = 0;
                if (cc < n_live) {
                    pm[cc] = __hip_atomic_load(a.part_m + pb + cc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    pl[cc] = __hip_atomic_load(a.part_l + pb + cc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                    for (int k = 0; k < EPT / 2; ++k)
                        po[cc][k] = __hip_atomic_load(reinterpret_cast<const uint64_t *>(a.part_o + (pb + cc) * HD + e0) + k,
                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            const int nc = a.row_pos[rr] / CT + 1;  // chunks that hold a position this row may see
            float M = -INFINITY;
#pragma unroll
            for (int cc = 0; cc < NCB; ++cc) M = cc < nc ? fmaxf(M, pm[cc]) : M;
            float L = 0.f, acc[EPT];
#pragma unroll
            for (int k = 0; k < EPT; ++k) acc[k] = 0.f;
#pragma unroll
            for (int cc = 0; cc < NCB; ++cc) {
                if (cc < nc) {
                    const float f = __expf(pm[cc] - M);
                    L += pl[cc] * f;
#pragma unroll
                    for (int k = 0; k < EPT / 2; ++k) {
                        acc[2 * k] += f32_lo(po[cc][k]) * f;
                        acc[2 * k + 1] += f32_hi(po[cc][k]) * f;
                    }
                }
            }
            const float inv = 1.f / L;
            const size_t o = ((size_t)rr * a.nq + hh) * HD + e0;
#pragma unroll
            for (int k = 0; k < EPT; k += 2) {
                const float v0 = acc[k] * inv, v1 = acc[k + 1] * inv;
                a.o[o + k] = v0;
                a.o[o + k + 1] = v1;
                const uint32_t hi = pack_bf16x2(v0, v1);
                *reinterpret_cast<uint32_t *>(a.ob + o + k) = hi;
                if (a.ob_lo)
                    *reinterpret_cast<uint32_t *>(a.ob + o + k + a.ob_lo) = pack_bf16x2(v0 - bf16_lo(hi), v1 - bf16_hi(hi));
            }
        }
    }
}

// ---- the same chunk streamed through three register buffers ---------------------------------------------------
// For passes whose attention launches thousands of workgroups (many sequences decoding in lock-step) a workgroup
// takes a long chunk (256 or 512 positions) and its waves walk their 16-position slabs w, w + 4, ... with the next
// two slabs' K rows and V columns in flight while this one is multiplied: the loads never pause for the arithmetic, and a
// sequence leaves two or three partials instead of a dozen.  The softmax runs on line: a wave keeps a running
// maximum per query, and rescales its sum and its output tile when a slab raises it.  The four waves' partials are
// merged as above.  One 16-query tile per workgroup: the tiles of a sequence run side by side in grid.z, each streaming
// the chunk for itself (the copies meet in the L2), rather than one after the other in one workgroup.
template <int HD>
__global__ __launch_bounds__(256, 2) void attn_stream_k(const AttnArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int ES = HD / 32, ET = HD / 16;
    const int CT = a.chunk;  // host: a multiple of 64
    const int QS = gridDim.z / a.batch;
    const int c = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z / QS, qs = blockIdx.z % QS;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int G = a.nq / a.kv.n_kv;
    const int r_first = a.row_off != nullptr ? a.row_off[b] : b * a.rps;
    const int rps = a.row_off != nullptr ? a.row_off[b + 1] - r_first : a.rps;
    if (rps <= 0) return;  // a sequence without rows in this pass (draft passes over the sequences still drafting)
    const int QN = G * rps;
    const int t0 = c * CT;
    const bf16_t *kp = reinterpret_cast<const bf16_t *>(a.kv.k);
    const bf16_t *vp = reinterpret_cast<const bf16_t *>(a.kv.v);

    __shared__ __attribute__((aligned(16))) float sO[4][16][HD + 4];
    __shared__ float sM[4][16], sL[4][16];

    const int cap = a.kv.pages_per_seq * a.kv.page_tokens;
    const bool has_qlo = a.qb_lo != 0;
    // the tiles of a sequence are shared out over grid.z / batch workgroups (the host launches one per tile of the
    // longest sequence, so that no workgroup streams its chunk more than once); a sequence with fewer tiles leaves
    // the others nothing to do
    const int QT = (QN + 15) / 16, TPW = (QT + QS - 1) / QS;
    const int qt_end = min(QT, (qs + 1) * TPW);
    if (qs * TPW >= qt_end) return;
    const int last_pos = __builtin_amdgcn_readfirstlane(a.row_pos[r_first + rps - 1]);
    if (t0 > last_pos) return;
    const int n_live = last_pos / CT + 1;
    // slabs of this chunk that hold a visible position (scalar: it bounds the loops around the matrix instructions)
    const int NS = (min(CT, last_pos - t0 + 1) + 15) >> 4;

    // Physical pages of the chunk's slabs, looked up once: a slab of 16 positions lies inside one page (host: pages
    // of at least 16 tokens), so the loads of a slab depend on nothing that is itself a load.  (Loads complete in
    // order: a block-table lookup per slab would make every wait for it wait for the slabs in flight as well.)
    __shared__ int s_page[32];
    if (threadIdx.x < 32) {
        const int pos = min(t0 + 16 * (int)threadIdx.x, cap - 1);
        s_page[threadIdx.x] = kv_page(a.kv, b, pos);
    }
    __syncthreads();
    const int pt_mask = a.kv.page_tokens - 1;
    const int k_step = kv_step_k(a.kv), v_step = kv_step_v(a.kv);
    struct Slab { u32x4_t kf[ES]; u32x2_t vf[ET]; };
    auto load_slab = [&](int sl, Slab &d) {
        const int tw = t0 + 16 * sl;
        const size_t base = kv_head_base(a.kv, s_page[sl], kvh);
        const int pk = min(tw + l16, cap - 1);
        const size_t kb = base + kv_in_k(a.kv, pk & pt_mask, 8 * g);
#pragma unroll
        for (int e = 0; e < ES; ++e) d.kf[e] = *reinterpret_cast<const u32x4_t *>(kp + kb + (size_t)e * k_step);
        const int pv = min(tw + 4 * g, cap - 4);
        const size_t vb = base + kv_in_v(a.kv, pv & pt_mask, l16);
#pragma unroll
        for (int et = 0; et < ET; ++et)
            d.vf[et] = *reinterpret_cast<const u32x2_t *>(vp + vb + (size_t)et * v_step);
    };

    for (int qt = qs * TPW; qt < qt_end; ++qt) {
        // Queries first, then the first two slabs, all before anything is waited for.  Every slab load below is
        // issued unconditionally (past the last slab the index is clamped, and the re-read hits the cache): the
        // number of loads in flight is then the same on every path through the loop, which is what lets the
        // waits before the matrix instructions leave the two younger slabs outstanding.
        const int qi = min(qt * 16 + l16, QN - 1);
        const int gq = qi / rps, qrow = r_first + qi % rps, qh = kvh * G + gq;
        const int qpos = a.row_pos[qrow];
        u32x4_t qf[ES], ql[ES];
        {
            const bf16_t *qp = a.qb + ((size_t)qrow * a.nq + qh) * HD + 8 * g;
#pragma unroll
            for (int e = 0; e < ES; ++e) {
                qf[e] = *reinterpret_cast<const u32x4_t *>(qp + 32 * e);
                ql[e] = has_qlo ? *reinterpret_cast<const u32x4_t *>(qp + a.qb_lo + 32 * e) : u32x4_t{0u, 0u, 0u, 0u};
            }
        }
        Slab A, B, C;
        load_slab(min(wave, NS - 1), A);
        load_slab(min(wave + 4, NS - 1), B);
        // a tile none of whose queries sees this chunk leaves no partial: the merge never reads one there
        if (t0 > __builtin_amdgcn_readfirstlane(wave_max(qpos))) continue;

        float m_run = -INFINITY, l_part = 0.f;
        f32x4_t O[ET];
#pragma unroll
        for (int et = 0; et < ET; ++et) O[et] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        auto process = [&](const Slab &d, int sl) {
            const int tw = t0 + 16 * sl;
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < ES; ++e) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, d.kf[e]),
                                                              __builtin_bit_cast(bf16x8_t, qf[e]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, d.kf[e]),
                                                              __builtin_bit_cast(bf16x8_t, ql[e]), acc, 0, 0, 0);
            }
            float sv[4], ms = -INFINITY;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                sv[v] = (tw + 4 * g + v) <= qpos ? acc[v] * a.scale : -INFINITY;
                ms = fmaxf(ms, sv[v]);
            }
            ms = fmaxf(ms, __shfl_xor(ms, 16, WAVE));
            ms = fmaxf(ms, __shfl_xor(ms, 32, WAVE));
            const float m_new = fmaxf(m_run, ms);
            // nothing visible yet: everything stays zero; first visible slab: the old (empty) state weighs nothing
            const float alpha = m_new == -INFINITY ? 1.f : (m_run == -INFINITY ? 0.f : __expf(m_run - m_new));
            float p[4], ps = 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                p[v] = m_new == -INFINITY ? 0.f : __expf(sv[v] - m_new);
                ps += p[v];
            }
            l_part = l_part * alpha + ps;
            m_run = m_new;
            // the output tile holds query 4 g + v in register v: its factor sits in the lane whose column is that query
            float aq[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) aq[v] = __shfl(alpha, 4 * g + v, WAVE);
            u32x2_t pw, pl;
            pw.x = pack_bf16x2(p[0], p[1]);
            pw.y = pack_bf16x2(p[2], p[3]);
            pl.x = pack_bf16x2(p[0] - bf16_lo(pw.x), p[1] - bf16_hi(pw.x));
            pl.y = pack_bf16x2(p[2] - bf16_lo(pw.y), p[3] - bf16_hi(pw.y));
#pragma unroll
            for (int et = 0; et < ET; ++et) {
#pragma unroll
                for (int v = 0; v < 4; ++v) O[et][v] *= aq[v];
                O[et] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, pw),
                                                                  __builtin_bit_cast(s16x4_t, d.vf[et]), O[et], 0, 0, 0);
                O[et] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, pl),
                                                                  __builtin_bit_cast(s16x4_t, d.vf[et]), O[et], 0, 0, 0);
            }
        };
        // three buffers in rotation: two slabs are in flight while one is multiplied
        for (int sl = wave; sl < NS; sl += 12) {
            load_slab(min(sl + 8, NS - 1), C);
            process(A, sl);
            load_slab(min(sl + 12, NS - 1), A);
            if (sl + 4 < NS) process(B, sl + 4);
            load_slab(min(sl + 16, NS - 1), B);
            if (sl + 8 < NS) process(C, sl + 8);
        }
        float l = l_part;
        l += __shfl_xor(l, 16, WAVE);
        l += __shfl_xor(l, 32, WAVE);
        if (g == 0) { sM[wave][l16] = m_run; sL[wave][l16] = l; }
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int v = 0; v < 4; ++v) sO[wave][4 * g + v][16 * et + l16] = O[et][v];
        __syncthreads();
        {
            constexpr int EPT = HD / 16;
            const int q = threadIdx.x >> 4, e0 = (threadIdx.x & 15) * EPT;
            const int qj = qt * 16 + q;
            if (qj < QN) {
                const float M = fmaxf(fmaxf(sM[0][q], sM[1][q]), fmaxf(sM[2][q], sM[3][q]));
                float f[4], L = 0.f, acc[EPT];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    f[w] = sM[w][q] == -INFINITY ? 0.f : __expf(sM[w][q] - M);
                    L += f[w] * sL[w][q];
                }
#pragma unroll
                for (int k = 0; k < EPT; ++k) acc[k] = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w)
#pragma unroll
                    for (int k = 0; k < EPT; ++k) acc[k] += f[w] * sO[w][q][e0 + k];
                const int rr = r_first + qj % rps, hh = kvh * G + qj / rps;
                if (n_live == 1) {
                    const size_t o = ((size_t)rr * a.nq + hh) * HD + e0;
#pragma unroll
                    for (int k = 0; k < EPT; ++k) {
                        const float v = acc[k] / L;
                        a.o[o + k] = v;
                        store_split_bf16(a.ob, o + k, a.ob_lo, v);
                    }
                } else {
                    const size_t pi = ((size_t)rr * a.nq + hh) * a.n_chunks + c;
                    float *po = a.part_o + pi * HD + e0;
#pragma unroll
                    for (int k = 0; k < EPT; ++k) po[k] = acc[k];
                    if (e0 == 0) { a.part_m[pi] = M; a.part_l[pi] = L; }
                }
            }
        }
        __syncthreads();
    }
}

// Merge of the chunk partials of the matrix-core kernel: o = sum_c w_c o_c with
// w_c = exp(m_c - M) / sum_c exp(m_c - M) l_c, in chunk order.  One thread per (row, head, four channels);
// rows of a sequence that fits one chunk were already written by attn_mfma_k.  The partials of all n_chunks
// chunks (NCB at most) are fetched at once, before the row's position says how many of them count, so that
// the kernel is one round of loads deep; chunks beyond the row's position hold stale finite numbers and are
// masked out.
template <int HD, int NCB>
__global__ __launch_bounds__(256) void attn_mfma_merge_k(const AttnArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int E4 = HD / 4;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.R * a.nq * E4) return;
    const int e = (idx % E4) * 4, hh = (idx / E4) % a.nq, rr = idx / (E4 * a.nq);
    const int b = a.row_off != nullptr ? a.row_seq[rr] : rr / a.rps;
    const size_t pb = ((size_t)rr * a.nq + hh) * a.n_chunks;
    float pm[NCB], pl[NCB];
    f32x4_t po[NCB];
#pragma unroll
    for (int cc = 0; cc < NCB; ++cc) {
        pm[cc] = -INFINITY; pl[cc] = 0.f; po[cc] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (cc < a.n_chunks) {
            pm[cc] = a.part_m[pb + cc];
            pl[cc] = a.part_l[pb + cc];
            po[cc] = *reinterpret_cast<const f32x4_t *>(a.part_o + (pb + cc) * HD + e);
        }
    }
    const int last_pos = a.row_pos[a.row_off != nullptr ? a.row_off[b + 1] - 1 : b * a.rps + a.rps - 1];
    if (last_pos / a.chunk == 0) return;
    const int nc = a.row_pos[rr] / a.chunk + 1;  // chunks that hold a position this row may see
    float M = -INFINITY;
#pragma unroll
    for (int cc = 0; cc < NCB; ++cc) M = cc < nc ? fmaxf(M, pm[cc]) : M;
    float L = 0.f;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cc = 0; cc < NCB; ++cc) {
        if (cc < nc) {
            const float f = __expf(pm[cc] - M);
            L += pl[cc] * f;
            acc[0] += po[cc][0] * f; acc[1] += po[cc][1] * f; acc[2] += po[cc][2] * f; acc[3] += po[cc][3] * f;
        }
    }
    const float inv = 1.f / L;
    acc[0] *= inv; acc[1] *= inv; acc[2] *= inv; acc[3] *= inv;
    const size_t o = ((size_t)rr * a.nq + hh) * HD + e;
    *reinterpret_cast<f32x4_t *>(a.o + o) = acc;
    u32x2_t ob;
    ob.x = pack_bf16x2(acc[0], acc[1]);
    ob.y = pack_bf16x2(acc[2], acc[3]);
    *reinterpret_cast<u32x2_t *>(a.ob + o) = ob;
    if (a.ob_lo) {
        u32x2_t lo;
        lo.x = pack_bf16x2(acc[0] - bf16_lo(ob.x), acc[1] - bf16_hi(ob.x));
        lo.y = pack_bf16x2(acc[2] - bf16_lo(ob.y), acc[3] - bf16_hi(ob.y));
        *reinterpret_cast<u32x2_t *>(a.ob + o + a.ob_lo) = lo;
    }
}

// Chunk size of the matrix-core kernel for a given capacity: 64 * 2^k positions, the smallest that keeps
// a sequence within 16 chunks (more, shorter chunks mean more workgroups but a longer merge).
int attention_mfma_chunk(int max_seq, int wanted) {
    if (wanted == 64 || wanted == 128 || wanted == 256 || wanted == 512) {
        if ((max_seq + wanted - 1) / wanted <= ATT_NC_MAX) return wanted;
    }
    int spw = 1;
    while (spw < ATT_SPW_MAX && (max_seq + 64 * spw - 1) / (64 * spw) > 16) spw *= 2;
    return 64 * spw;
}

bool attention_uses_mfma(const AttnArgs &a, int hd) {
    return a.kv_dtype == DT_BF16 && a.qb != nullptr && a.kv.page_tokens % 4 == 0 &&
           (hd == 32 || hd == 64 || hd == 128);
}

template <int HD>
static hipError_t launch_attn_mfma(const AttnArgs &a, dim3 grid, hipStream_t s) {
    if (a.stream_chunks) {
        hipLaunchKernelGGL((attn_stream_k<HD>), grid, dim3(256), 0, s, a);
        const hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess || a.n_chunks == 1) return e0;
        const int items0 = a.R * a.nq * (HD / 4);
        if (a.n_chunks <= 16) hipLaunchKernelGGL((attn_mfma_merge_k<HD, 16>), dim3((items0 + 255) / 256), dim3(256), 0, s, a);
        else hipLaunchKernelGGL((attn_mfma_merge_k<HD, ATT_NC_MAX>), dim3((items0 + 255) / 256), dim3(256), 0, s, a);
        return hipGetLastError();
    }
    // queries held ahead: chunks of up to 128 positions (beyond, the K / V fragments leave no registers) and few
    // enough workgroups that a compute unit does not wait for a slot
    const bool ahead = a.chunk <= 128 && (size_t)grid.x * grid.y * grid.z <= 1024;
    // The fused merge: few workgroups, at most eight queries per (sequence, kv head) - decode rows - and no more chunks
    // than it holds at once.  Measured on the 8B-shaped pair: the draft's attention (4 queries) 12.2 -> 10.8 us per
    // layer including the launch gaps, the target's verification (16 queries) 14.6 -> 15.9 us, so that one keeps the
    // second kernel.
    static const bool no_fuse = std::getenv("SPEC_NO_ATTN_FUSE") != nullptr;
    const bool fuse = ahead && !no_fuse && a.ticket != nullptr && (int)grid.z == a.batch && a.row_off == nullptr &&
                      a.nq / a.kv.n_kv * a.rps <= 8 && a.n_chunks > 1 && a.n_chunks <= 16;
    switch (a.chunk / 64) {
        case 1:
            if (fuse) hipLaunchKernelGGL((attn_mfma_k<HD, 1, true, true>), grid, dim3(256), 0, s, a);
            else if (ahead) hipLaunchKernelGGL((attn_mfma_k<HD, 1, true>), grid, dim3(256), 0, s, a);
            else hipLaunchKernelGGL((attn_mfma_k<HD, 1, false>), grid, dim3(256), 0, s, a);
            break;
        case 2:
            if (fuse) hipLaunchKernelGGL((attn_mfma_k<HD, 2, true, true>), grid, dim3(256), 0, s, a);
            else if (ahead) hipLaunchKernelGGL((attn_mfma_k<HD, 2, true>), grid, dim3(256), 0, s, a);
            else hipLaunchKernelGGL((attn_mfma_k<HD, 2, false>), grid, dim3(256), 0, s, a);
            break;
        case 4: hipLaunchKernelGGL((attn_mfma_k<HD, 4, false>), grid, dim3(256), 0, s, a); break;
        default: hipLaunchKernelGGL((attn_mfma_k<HD, 8, false>), grid, dim3(256), 0, s, a); break;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.n_chunks == 1 || fuse) return e;
    const int items = a.R * a.nq * (HD / 4);
    if (a.n_chunks <= 16) hipLaunchKernelGGL((attn_mfma_merge_k<HD, 16>), dim3((items + 255) / 256), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((attn_mfma_merge_k<HD, ATT_NC_MAX>), dim3((items + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

// a.chunk / a.n_chunks: 64 and ceil(max_seq / 64) for the plain kernel, attention_mfma_chunk() and the
// matching count for the matrix-core kernel.
hipError_t launch_attention(const AttnArgs &a, int hd, hipStream_t s) {
    const int B = a.batch;
    if (a.row_off != nullptr && !attention_uses_mfma(a, hd)) return hipErrorInvalidValue;  // ragged rows: matrix-core kernels only
    if (attention_uses_mfma(a, hd)) {
        const int spw = a.chunk / 64;
        if (a.chunk % 64 || (spw != 1 && spw != 2 && spw != 4 && spw != 8) || a.n_chunks > ATT_NC_MAX)
            return hipErrorInvalidValue;
        const int QT = (a.nq / a.kv.n_kv * a.rps + 15) / 16;
        // streamed chunks: a workgroup per tile (a second tile would stream the chunk a second time, one after the other)
        const int tpw = a.stream_chunks ? 1 : ATT_TILES_PER_WG;
        const dim3 grid(a.n_chunks, a.kv.n_kv, B * ((QT + tpw - 1) / tpw));
        if (hd == 32) return launch_attn_mfma<32>(a, grid, s);
        if (hd == 64) return launch_attn_mfma<64>(a, grid, s);
        return launch_attn_mfma<128>(a, grid, s);
    }
    if (a.rps > ATT_RPS_MAX || a.chunk != ATT_CT) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_simple_k, dim3(a.n_chunks, a.nq, B), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_combine_k, dim3(a.R, a.nq), dim3(128), 0, s, a);
    return hipGetLastError();
}

}  // namespace sd
