// Attention of the rows of one forward pass against the paged KV cache, split over KV chunks
// (partial softmax per chunk, merged by a combine kernel).  The rows of a sequence are the
// gamma+1 verification rows of the target, or the 1-2 decode rows of the draft; row i may see
// cache positions <= its own position (causal inside the rows).
//
// attn_simple_k is the plain version: any head size and cache type, fp32 arithmetic, one
// workgroup per (chunk, query head, sequence).  It serves fp32 models.
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
            const size_t kb = kv_index_k(a.kv, b, pos, kvh, 0);
            float acc = 0.f;
            for (int e = 0; e < hd; ++e) acc = fmaf(q[e], kv_load(a.kv.k, a.kv_dtype, kb + e), acc);
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
// One workgroup per (chunk of 64 * spw positions, kv head, sequence); wave w owns the 16-position slabs
// w, w + 4, ... of the chunk.  Per 16-query tile a wave forms S^T = K Q^T with
// v_mfma_f32_16x16x32_bf16 (K rows and bf16 query rows are loaded straight into the operand layout),
// takes the softmax over its slabs, and multiplies by V with v_mfma_f32_16x16x16_bf16: the S^T result
// registers already are the A operand (query = lane % 16, four positions per lane), and the transposed
// V pages give the B operand with one 8-byte load.  The four wave partials are merged through LDS into
// one (max, sum, vector) partial per chunk; the workgroup that finishes last for its (sequence, kv head)
// merges the chunk partials, in chunk order, into the attention output.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int ATT_SPW_MAX = 8;  // slabs per wave -> chunks of up to 512 positions

template <int HD>
__global__ __launch_bounds__(256) void attn_mfma_k(const AttnArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int ES = HD / 32;  // k-steps of the score product
    constexpr int ET = HD / 16;  // 16-channel tiles of the output
    const int c = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    // wave index and last position are scalars: branches around matrix instructions must be scalar
    // branches, since v_mfma ignores the execution mask
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int G = a.nq / a.kv.n_kv;
    const int QN = G * a.rps;
    const int r_first = b * a.rps;
    const int CT = a.chunk, spw = a.chunk >> 6;
    const int t0 = c * CT;
    const int last_pos = __builtin_amdgcn_readfirstlane(a.row_pos[r_first + a.rps - 1]);
    if (t0 > last_pos) return;
    const bf16_t *kp = reinterpret_cast<const bf16_t *>(a.kv.k);
    const bf16_t *vp = reinterpret_cast<const bf16_t *>(a.kv.v);

    __shared__ float sO[4][16][HD + 1];
    __shared__ float sM[4][16], sL[4][16];
    __shared__ int s_last;

    const int QT = (QN + 15) / 16;
    for (int qt = 0; qt < QT; ++qt) {
        // query handled by this lane in the score product (column l16 of S^T)
        const int qi = min(qt * 16 + l16, QN - 1);
        const int gq = qi / a.rps, i = qi % a.rps;
        const int r = r_first + i, h = kvh * G + gq;
        const int qpos = a.row_pos[r];
        u32x4_t qf[ES];
        {
            const bf16_t *qp = a.qb + ((size_t)r * a.nq + h) * HD + 8 * g;
#pragma unroll
            for (int s = 0; s < ES; ++s) qf[s] = *reinterpret_cast<const u32x4_t *>(qp + 32 * s);
        }
        // pass 1: scores of every slab of this wave; S[sl][v] = (position tw + 4 g + v, query l16)
        f32x4_t S[ATT_SPW_MAX];
        float m = -INFINITY;
#pragma unroll
        for (int sl = 0; sl < ATT_SPW_MAX; ++sl) {
            S[sl] = f32x4_t{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            const int tw = t0 + 16 * (wave + 4 * sl);
            if (sl < spw && tw <= last_pos) {
                const int pos = min(tw + l16, last_pos);
                const size_t kb = kv_index_k(a.kv, b, pos, kvh, 0);
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < ES; ++s) {
                    const u32x4_t kf = *reinterpret_cast<const u32x4_t *>(kp + kb + 32 * s + 8 * g);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf),
                                                                  __builtin_bit_cast(bf16x8_t, qf[s]), acc, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const bool vis = (tw + 4 * g + v) <= qpos;
                    S[sl][v] = vis ? acc[v] * a.scale : -INFINITY;
                    m = fmaxf(m, S[sl][v]);
                }
            }
        }
        m = fmaxf(m, __shfl_xor(m, 16, WAVE));
        m = fmaxf(m, __shfl_xor(m, 32, WAVE));
        // pass 2: probabilities and the weighted values
        float l = 0.f;
        f32x4_t O[ET];
#pragma unroll
        for (int et = 0; et < ET; ++et) O[et] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sl = 0; sl < ATT_SPW_MAX; ++sl) {
            const int tw = t0 + 16 * (wave + 4 * sl);
            if (sl < spw && tw <= last_pos) {
                float p[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    p[v] = m == -INFINITY ? 0.f : __expf(S[sl][v] - m);
                    l += p[v];
                }
                u32x2_t pw;
                pw.x = pack_bf16x2(p[0], p[1]);
                pw.y = pack_bf16x2(p[2], p[3]);
                // V fragment: channel 16 et + l16, positions tw + 4 g .. + 4 (contiguous in the transposed page)
                const int pos = min(tw + 4 * g, last_pos & ~3);
#pragma unroll
                for (int et = 0; et < ET; ++et) {
                    const u32x2_t vf = *reinterpret_cast<const u32x2_t *>(vp + kv_index_v(a.kv, b, pos, kvh, 16 * et + l16));
                    O[et] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, pw),
                                                                      __builtin_bit_cast(s16x4_t, vf), O[et], 0, 0, 0);
                }
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
        // merge the four wave partials: thread -> (query, channel)
        for (int idx = threadIdx.x; idx < 16 * HD; idx += 256) {
            const int q = idx / HD, e = idx % HD;
            const int qj = qt * 16 + q;
            if (qj >= QN) continue;
            const float M = fmaxf(fmaxf(sM[0][q], sM[1][q]), fmaxf(sM[2][q], sM[3][q]));
            float acc = 0.f, L = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float f = sM[w][q] == -INFINITY ? 0.f : __expf(sM[w][q] - M);
                acc += f * sO[w][q][e];
                L += f * sL[w][q];
            }
            const int rr = r_first + qj % a.rps, hh = kvh * G + qj / a.rps;
            const size_t pi = ((size_t)rr * a.nq + hh) * a.n_chunks + c;
            a.part_o[pi * HD + e] = acc;
            if (e == 0) { a.part_m[pi] = M; a.part_l[pi] = L; }
        }
        __syncthreads();
    }

    // the last workgroup of this (sequence, kv head) merges the chunk partials; every thread publishes
    // its own partial stores before the arrival is counted
    const int n_live = last_pos / CT + 1;
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t t = atomicAdd(&a.cnt[b * a.kv.n_kv + kvh], 1u);
        s_last = (t == (uint32_t)(n_live - 1));
        if (s_last) a.cnt[b * a.kv.n_kv + kvh] = 0;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    const volatile float *pm = a.part_m, *pl = a.part_l, *po = a.part_o;
    for (int idx = threadIdx.x; idx < QN * HD; idx += 256) {
        const int qj = idx / HD, e = idx % HD;
        const int rr = r_first + qj % a.rps, hh = kvh * G + qj / a.rps;
        const int nc = a.row_pos[rr] / CT + 1;  // chunks that hold a position this row may see
        const size_t pb = ((size_t)rr * a.nq + hh) * a.n_chunks;
        float M = -INFINITY;
        for (int cc = 0; cc < nc; ++cc) M = fmaxf(M, pm[pb + cc]);
        float L = 0.f, acc = 0.f;
        for (int cc = 0; cc < nc; ++cc) {
            const float f = __expf(pm[pb + cc] - M);
            L += pl[pb + cc] * f;
            acc += po[(pb + cc) * HD + e] * f;
        }
        const float v = acc / L;
        const size_t o = ((size_t)rr * a.nq + hh) * HD + e;
        a.o[o] = v;
        a.ob[o] = f32_to_bf16(v);
    }
}

// Chunk size (a multiple of 64 positions) of the matrix-core kernel for a given capacity: at most eight
// chunks per sequence while the capacity allows it.
int attention_mfma_chunk(int max_seq) {
    int spw = (max_seq + 64 * 8 - 1) / (64 * 8);
    if (spw < 1) spw = 1;
    if (spw > ATT_SPW_MAX) spw = ATT_SPW_MAX;
    return 64 * spw;
}

bool attention_uses_mfma(const AttnArgs &a, int hd) {
    return a.kv_dtype == DT_BF16 && a.qb != nullptr && a.cnt != nullptr && a.kv.page_tokens % 4 == 0 &&
           (hd == 32 || hd == 64 || hd == 128);
}

// a.chunk / a.n_chunks: 64 and ceil(max_seq / 64) for the plain kernel, attention_mfma_chunk() and the
// matching count for the matrix-core kernel.
hipError_t launch_attention(const AttnArgs &a, int hd, hipStream_t s) {
    const int B = a.R / a.rps;
    if (attention_uses_mfma(a, hd)) {
        if (a.chunk % 64 || a.chunk < 64 || a.chunk > 64 * ATT_SPW_MAX) return hipErrorInvalidValue;
        const dim3 grid(a.n_chunks, a.kv.n_kv, B);
        if (hd == 32) hipLaunchKernelGGL(attn_mfma_k<32>, grid, dim3(256), 0, s, a);
        else if (hd == 64) hipLaunchKernelGGL(attn_mfma_k<64>, grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL(attn_mfma_k<128>, grid, dim3(256), 0, s, a);
        return hipGetLastError();
    }
    if (a.rps > ATT_RPS_MAX || a.chunk != ATT_CT) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_simple_k, dim3(a.n_chunks, a.nq, B), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_combine_k, dim3(a.R, a.nq), dim3(128), 0, s, a);
    return hipGetLastError();
}

}  // namespace sd
