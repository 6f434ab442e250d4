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
// One workgroup per (64-position chunk, kv head, sequence); each of its four waves owns 16 positions.
// Per 16-query tile a wave forms S^T = K Q^T with v_mfma_f32_16x16x32_bf16 (K rows and bf16 query rows
// are loaded straight into the operand layout), takes the slab-local softmax, and multiplies by V with
// v_mfma_f32_16x16x16_bf16: the S^T result registers already are the A operand (query = lane % 16,
// four positions per lane), and the transposed V pages give the B operand with one 8-byte load.
// K and V fragments of the slab stay in registers across query tiles.  The four slab partials are
// merged through LDS, so one (max, sum, vector) partial per chunk reaches the combine kernel.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

template <int HD>
__global__ __launch_bounds__(256) void attn_mfma_k(const AttnArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int ES = HD / 32;  // k-steps of the score product
    constexpr int ET = HD / 16;  // 16-channel tiles of the output
    const int c = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int G = a.nq / a.kv.n_kv;
    const int QN = G * a.rps;
    const int r_first = b * a.rps;
    const int t0 = c * ATT_CT;
    const int last_pos = a.row_pos[r_first + a.rps - 1];
    if (t0 > last_pos) return;
    const int t0w = t0 + 16 * wave;
    const bool slab_live = t0w <= last_pos;
    const bf16_t *kp = reinterpret_cast<const bf16_t *>(a.kv.k);
    const bf16_t *vp = reinterpret_cast<const bf16_t *>(a.kv.v);

    // K fragment: row = position t0w + l16, channels 32 s + 8 g .. + 8
    u32x4_t kf[ES];
    {
        const int pos = min(t0w + l16, last_pos);
        const size_t kb = kv_index_k(a.kv, b, pos, kvh, 0);
#pragma unroll
        for (int s = 0; s < ES; ++s) kf[s] = *reinterpret_cast<const u32x4_t *>(kp + kb + 32 * s + 8 * g);
    }
    // V fragment: channel 16 et + l16, positions t0w + 4 g .. + 4 (contiguous in the transposed page)
    u32x2_t vf[ET];
    {
        const int pos = min(t0w + 4 * g, last_pos & ~3);
#pragma unroll
        for (int et = 0; et < ET; ++et)
            vf[et] = *reinterpret_cast<const u32x2_t *>(vp + kv_index_v(a.kv, b, pos, kvh, 16 * et + l16));
    }

    __shared__ float sO[4][16][HD + 1];
    __shared__ float sM[4][16], sL[4][16];

    const int QT = (QN + 15) / 16;
    for (int qt = 0; qt < QT; ++qt) {
        // query handled by this lane in the score product (column l16 of S^T)
        const int qi = min(qt * 16 + l16, QN - 1);
        const int gq = qi / a.rps, i = qi % a.rps;
        const int r = r_first + i, h = kvh * G + gq;
        f32x4_t S = {0.f, 0.f, 0.f, 0.f};
        if (slab_live) {
            const bf16_t *qp = a.qb + ((size_t)r * a.nq + h) * HD + 8 * g;
#pragma unroll
            for (int s = 0; s < ES; ++s) {
                const u32x4_t qf = *reinterpret_cast<const u32x4_t *>(qp + 32 * s);
                S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[s]),
                                                            __builtin_bit_cast(bf16x8_t, qf), S, 0, 0, 0);
            }
        }
        // S[v] = score of (position t0w + 4 g + v, query l16)
        const int qpos = a.row_pos[r];
        float m = -INFINITY;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const bool vis = slab_live && (t0w + 4 * g + v) <= qpos;
            S[v] = vis ? S[v] * a.scale : -INFINITY;
            m = fmaxf(m, S[v]);
        }
        m = fmaxf(m, __shfl_xor(m, 16, WAVE));
        m = fmaxf(m, __shfl_xor(m, 32, WAVE));
        float p[4], l = 0.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            p[v] = m == -INFINITY ? 0.f : __expf(S[v] - m);
            l += p[v];
        }
        l += __shfl_xor(l, 16, WAVE);
        l += __shfl_xor(l, 32, WAVE);
        u32x2_t pw;
        pw.x = pack_bf16x2(p[0], p[1]);
        pw.y = pack_bf16x2(p[2], p[3]);
        if (g == 0) { sM[wave][l16] = m; sL[wave][l16] = l; }
        // O tile et: result register v of lane (channel l16, g) is query 4 g + v
#pragma unroll
        for (int et = 0; et < ET; ++et) {
            f32x4_t O = {0.f, 0.f, 0.f, 0.f};
            O = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, pw),
                                                          __builtin_bit_cast(s16x4_t, vf[et]), O, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) sO[wave][4 * g + v][16 * et + l16] = O[v];
        }
        __syncthreads();
        // merge the four slabs: thread -> (query, channel stripe)
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
}

hipError_t launch_attention(const AttnArgs &a, int hd, hipStream_t s) {
    if (a.rps > ATT_RPS_MAX || a.chunk != ATT_CT) return hipErrorInvalidValue;
    const int B = a.R / a.rps;
    const bool mfma = a.kv_dtype == DT_BF16 && a.qb != nullptr && a.kv.page_tokens % 4 == 0 &&
                      (hd == 32 || hd == 64 || hd == 128);
    if (mfma) {
        const dim3 grid(a.n_chunks, a.kv.n_kv, B);
        if (hd == 32) hipLaunchKernelGGL(attn_mfma_k<32>, grid, dim3(256), 0, s, a);
        else if (hd == 64) hipLaunchKernelGGL(attn_mfma_k<64>, grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL(attn_mfma_k<128>, grid, dim3(256), 0, s, a);
    } else {
        hipLaunchKernelGGL(attn_simple_k, dim3(a.n_chunks, a.nq, B), dim3(256), 0, s, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_combine_k, dim3(a.R, a.nq), dim3(128), 0, s, a);
    return hipGetLastError();
}

}  // namespace sd
