// Small kernels around the projections: step bookkeeping, token embedding, weight re-tiling,
// seeded fills, and a Philox probe for parity tests.
#include "common.hpp"
#include "kv.hpp"
#include "params.hpp"

namespace sd {

// Start of the draft phase of a speculative step: advance the step ordinal, mark every sequence as
// drafting, and fetch the planned gamma of each sequence (gamma_plan: device-visible host memory,
// written by the host before the launch).
__global__ void begin_draft_k(State st, const int32_t *gamma_plan) {
    const int b = threadIdx.x;
    if (b == 0) {
        st.ctl[0] += 1;
        st.ctl[1] = st.batch;
    }
    if (b < st.batch) {
        st.k[b] = 0;
        st.gamma_b[b] = gamma_plan[b];
    }
}

hipError_t launch_begin_draft(const State &st, const int32_t *gamma_plan, hipStream_t s) {
    if (st.batch > 256) return hipErrorInvalidValue;
    hipLaunchKernelGGL(begin_draft_k, dim3(1), dim3(256), 0, s, st, gamma_plan);
    return hipGetLastError();
}

__device__ __forceinline__ int row_position(const State &st, const RowPlan &p, int b, int i) {
    switch (p.mode) {
        case ROWS_PREFILL: return p.arg + i;
        case ROWS_VERIFY: return st.len[b] - 1 + i;
        case ROWS_DRAFT_FIRST: return max(st.len[b] - 2 + i, 0);
        default: return st.len[b] + p.arg - 2;  // ROWS_DRAFT_NEXT: the token drafted one step earlier
    }
}

// One workgroup per row: look the token up, copy its embedding into the fp32 residual stream,
// emit the row scaled by the first norm weight (fp32 and bf16) and its sum of squares.
__global__ __launch_bounds__(256) void embed_k(const EmbedArgs a) {
    if (a.plan.mode == ROWS_DRAFT_NEXT && a.st.ctl[1] == 0) return;
    const int r = blockIdx.x;
    int b = r / a.plan.rps, i = r % a.plan.rps;
    if (a.plan.ragged && a.plan.mode == ROWS_DRAFT_NEXT) {
        // row r belongs to the r-th sequence that still drafts (a scan over at most 64 sequences); a row past their
        // number (the host counted them) repeats the last one
        int seen = 0;
        b = 0;
        for (int s = 0; s < a.st.batch; ++s) {
            if (a.st.k[s] == 0) {
                if (seen <= r) b = s;
                ++seen;
            }
        }
        i = 0;
        if (r == 0 && threadIdx.x == 0) {
            int o = 0;
            for (int s = 0; s < a.st.batch; ++s) { a.row_off[s] = o; o += a.st.k[s] == 0; }
            a.row_off[a.st.batch] = o;
        }
    } else if (a.plan.ragged) {
        // sequence b owns rows off_b .. off_b + gamma_b[b]: a scan over at most 64 sequences
        int off = 0;
        b = 0;
        while (b + 1 < a.st.batch && r >= off + a.st.gamma_b[b] + 1) off += a.st.gamma_b[b++] + 1;
        i = r - off;
        if (r == 0 && threadIdx.x == 0) {
            int o = 0;
            for (int s = 0; s < a.st.batch; ++s) { a.row_off[s] = o; o += a.st.gamma_b[s] + 1; }
            a.row_off[a.st.batch] = o;
        }
    }
    int pos = row_position(a.st, a.plan, b, i);
    pos = min(max(pos, 0), a.st.max_seq - 1);
    int tok = a.st.tokens[(size_t)b * a.st.max_seq + pos];
    tok = min(max(tok, 0), a.vocab - 1);
    if (threadIdx.x == 0) {
        a.row_pos[r] = pos;
        a.row_seq[r] = b;
    }
    float ss = 0.f;
    for (int c = threadIdx.x; c < a.d; c += 256) {
        float v;
        if (a.dtype == DT_BF16) v = bf16_to_f32(reinterpret_cast<const bf16_t *>(a.embed)[(size_t)tok * a.d + c]);
        else v = reinterpret_cast<const float *>(a.embed)[(size_t)tok * a.d + c];
        const float g = a.g_next[c];
        const size_t o = (size_t)r * a.d + c;
        a.x[o] = v;
        a.xg[o] = v * g;
        store_split_bf16(a.xgb, o, a.xgb_lo, v * g);
        ss += v * v;
    }
    __shared__ float red[4];
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) a.ssq_out[(size_t)r * a.ssq_stride] = red[0] + red[1] + red[2] + red[3];
}

hipError_t launch_embed(const EmbedArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(embed_k, dim3(a.R), dim3(256), 0, s, a);
    return hipGetLastError();
}

// Row-major bf16 -> 16-row groups of 1 KiB tiles.  Tile (group g, k-tile t) holds, for lane l, the 8
// values of packed row 16 g + l % 16 at k = 32 t + 8 (l / 16) .. +8; tiles of a group are contiguous in t.
// Packed rows of the fused matrices are ordered so that an epilogue finds both partners of a pair in
// one group: rows 0-7 of a group are first elements (gate rows, or RoPE elements j), rows 8-15 the
// matching second elements (up rows, or RoPE elements j + hd/2).
// Packed row p -> (source matrix 0..2, row in it).
__device__ __forceinline__ void retile_source(const RetileArgs &a, int p, int &which, int &row) {
    which = 0;
    row = p;
    if (a.mode == EPI_SWIGLU) {
        const int gi = p >> 4, pos = p & 15;
        row = gi * 8 + (pos & 7);
        which = pos < 8 ? 0 : 1;
    } else if (a.mode == EPI_QKV) {
        const int half = a.hd >> 1;
        const int gi = p >> 4, pos = p & 15;
        const int P = gi * 8 + (pos & 7);
        int hh = P / half;
        const int j = P % half + (pos < 8 ? 0 : half);
        if (hh >= a.nq + a.nkv) { which = 2; hh -= a.nq + a.nkv; }
        else if (hh >= a.nq) { which = 1; hh -= a.nq; }
        row = hh * a.hd + j;
    }
}

__global__ __launch_bounds__(256) void retile_k(const RetileArgs a, uint4 *__restrict__ out) {
    // 16-bit weights: tiles of 16 rows x 32 k; 8-bit weights: 16 rows x 64 k.  Either way lane l of a tile holds 16
    // bytes of row l % 16: k-chunk l / 16 of four.
    const int esz = a.q8 ? 1 : 2, tk = a.q8 ? 64 : 32;
    const int KT = a.K / tk;
    const int64_t total = (int64_t)(a.Ntot / 16) * KT * 64;
    const char *base[3] = {reinterpret_cast<const char *>(a.w0), reinterpret_cast<const char *>(a.w1),
                           reinterpret_cast<const char *>(a.w2)};
    for (int64_t idx = blockIdx.x * (int64_t)256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int l = (int)(idx & 63);
        const int64_t tile = idx >> 6;
        const int t = (int)(tile % KT);
        const int g = (int)(tile / KT);
        int which, row;
        retile_source(a, g * 16 + (l & 15), which, row);
        const char *src = (which == 0 ? base[0] : (which == 1 ? base[1] : base[2])) +
                          ((size_t)row * a.K + (size_t)t * tk + (l >> 4) * (tk / 4)) * esz;
        out[idx] = *reinterpret_cast<const uint4 *>(src);
    }
    // the per-row scales of 8-bit weights, in packed row order
    if (a.q8 && a.scale_out != nullptr) {
        const float *sc[3] = {a.s0, a.s1, a.s2};
        for (int p = blockIdx.x * 256 + threadIdx.x; p < a.Ntot; p += gridDim.x * 256) {
            int which, row;
            retile_source(a, p, which, row);
            a.scale_out[p] = (which == 0 ? sc[0] : (which == 1 ? sc[1] : sc[2]))[row];
        }
    }
}

hipError_t launch_retile(const RetileArgs &a, void *out, hipStream_t s) {
    if (a.Ntot % 16 != 0 || a.K % (a.q8 ? 64 : 32) != 0) return hipErrorInvalidValue;
    if (a.mode == EPI_QKV && ((a.hd / 2) % 8 != 0)) return hipErrorInvalidValue;
    if (a.mode == EPI_SWIGLU && (a.Ntot / 2) % 8 != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(retile_k, dim3(4096), dim3(256), 0, s, a, reinterpret_cast<uint4 *>(out));
    return hipGetLastError();
}

__global__ void philox_k(uint64_t seed, const uint32_t *ctr, int n, uint32_t *out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const Philox4 r = philox4x32_10(ctr[4 * i], ctr[4 * i + 1], ctr[4 * i + 2], ctr[4 * i + 3], (uint32_t)seed,
                                    (uint32_t)(seed >> 32));
    for (int j = 0; j < 4; ++j) out[4 * i + j] = r.v[j];
}

hipError_t launch_philox(uint64_t seed, const uint32_t *ctr, int n, uint32_t *out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(philox_k, dim3((n + 255) / 256), dim3(256), 0, s, seed, ctr, n, out);
    return hipGetLastError();
}

// Seeded values in [-1, 1) (synthetic KV contents for verify-only sweeps).
__global__ void fill_uniform_k(void *dst, int64_t n, int dtype, uint64_t seed) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const Philox4 r = philox4x32_10((uint32_t)i, (uint32_t)(i >> 32), 0x4b56u, 0, (uint32_t)seed, (uint32_t)(seed >> 32));
        const float v = (float)(r.v[0] >> 8) * (2.0f / 16777216.0f) - 1.0f;
        if (dtype == DT_BF16) reinterpret_cast<bf16_t *>(dst)[i] = f32_to_bf16(v);
        else reinterpret_cast<float *>(dst)[i] = v;
    }
}

hipError_t launch_fill_uniform(void *dst, int64_t n, int dtype, uint64_t seed, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_uniform_k, dim3(4096), dim3(256), 0, s, dst, n, dtype, seed);
    return hipGetLastError();
}

__global__ void cast_to_f32_k(const void *src, int dtype, float *dst, int64_t n) {
    const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i >= n) return;
    dst[i] = dtype == DT_BF16 ? bf16_to_f32(reinterpret_cast<const bf16_t *>(src)[i])
                              : reinterpret_cast<const float *>(src)[i];
}

// dst[i] = bf16(src[i]); with lo_off != 0 also dst[lo_off + i] = bf16(src[i] - dst[i])
__global__ void cast_to_bf16_k(const float *src, uint16_t *dst, int64_t lo_off, int64_t n) {
    const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i < n) store_split_bf16(dst, (size_t)i, lo_off, src[i]);
}

hipError_t launch_cast_to_bf16(const float *src, uint16_t *dst, int64_t lo_off, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(cast_to_bf16_k, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, dst, lo_off, n);
    return hipGetLastError();
}

hipError_t launch_cast_to_f32(const void *src, int dtype, float *dst, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(cast_to_f32_k, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, dtype, dst, n);
    return hipGetLastError();
}

// Write caller-supplied K / V rows [n][n_kv][hd] (fp32) of one sequence into the paged cache at positions pos0...
__global__ __launch_bounds__(256) void kv_write_k(KVCache kv, int kv_dtype, int seq, int pos0, int n, const float *k,
                                                   const float *v) {
    const int64_t total = (int64_t)n * kv.n_kv * kv.hd;
    for (int64_t i = blockIdx.x * (int64_t)256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int j = (int)(i % kv.hd);
        const int h = (int)((i / kv.hd) % kv.n_kv);
        const int t = (int)(i / ((int64_t)kv.hd * kv.n_kv));
        kv_store(kv, kv_dtype, true, seq, pos0 + t, h, j, k[i]);
        kv_store(kv, kv_dtype, false, seq, pos0 + t, h, j, v[i]);
    }
}

hipError_t launch_kv_write(const KVCache &kv, int kv_dtype, int seq, int pos0, int n, const float *k, const float *v,
                           hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(kv_write_k, dim3(1024), dim3(256), 0, s, kv, kv_dtype, seq, pos0, n, k, v);
    return hipGetLastError();
}

// Plain copy, 16 bytes per lane (the reference point that scales the profiler's HBM byte counters).
__global__ __launch_bounds__(256) void copy_k(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n16) {
    for (int64_t i = blockIdx.x * (int64_t)256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy(const void *src, void *dst, int64_t bytes, hipStream_t s) {
    if (bytes <= 0) return hipSuccess;
    if (bytes % 16) return hipErrorInvalidValue;
    const int64_t n16 = bytes / 16;
    const int64_t blocks = (n16 + 255) / 256;
    hipLaunchKernelGGL(copy_k, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, s,
                       reinterpret_cast<const uint4 *>(src), reinterpret_cast<uint4 *>(dst), n16);
    return hipGetLastError();
}

}  // namespace sd
