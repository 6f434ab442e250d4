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

hipError_t launch_attention(const AttnArgs &a, int hd, hipStream_t s) {
    (void)hd;
    if (a.rps > ATT_RPS_MAX || a.chunk != ATT_CT) return hipErrorInvalidValue;
    const int B = a.R / a.rps;
    hipLaunchKernelGGL(attn_simple_k, dim3(a.n_chunks, a.nq, B), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_combine_k, dim3(a.R, a.nq), dim3(128), 0, s, a);
    return hipGetLastError();
}

}  // namespace sd
