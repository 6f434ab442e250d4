// Epilogues of the fused projections, applied by a whole workgroup to its reduced output tile.
//
// The tile holds R rows x TW "packed" output columns in LDS (row-major, row stride TS).  Packed
// columns are ordered so that both partners of a pair sit in one tile: columns [0, TW/2) are first
// elements (gate rows, RoPE elements j), columns [TW/2, TW) the matching second elements (up rows,
// RoPE elements j + hd/2).  For plain / residual / logits tiles packed column c of tile t is output
// column t * TW + c.
#pragma once

#include "common.hpp"
#include "kv.hpp"
#include "params.hpp"

namespace sd {

// Weight row (in the caller's row-major matrices) behind packed row p, for tiles of TW packed rows.
template <typename WT, int EPI>
__device__ __forceinline__ const WT *packed_row(const GemvArgs &a, int p, int TW) {
    if constexpr (EPI == EPI_SWIGLU) {
        const int h2 = TW >> 1;
        const int gi = p / TW, pos = p % TW;
        const int j = gi * h2 + pos % h2;
        const WT *base = reinterpret_cast<const WT *>(pos < h2 ? a.w0 : a.w1);
        return base + (size_t)j * a.K;
    } else if constexpr (EPI == EPI_QKV) {
        const int h2 = TW >> 1;
        const int half = a.hd >> 1;
        const int gi = p / TW, pos = p % TW;
        const int P = gi * h2 + pos % h2;
        int hh = P / half;
        const int j = P % half + (pos < h2 ? 0 : half);
        const WT *base = reinterpret_cast<const WT *>(a.w0);
        if (hh >= a.nq + a.nkv) { base = reinterpret_cast<const WT *>(a.w2); hh -= a.nq + a.nkv; }
        else if (hh >= a.nq) { base = reinterpret_cast<const WT *>(a.w1); hh -= a.nq; }
        return base + ((size_t)hh * a.hd + j) * a.K;
    } else {
        return reinterpret_cast<const WT *>(a.w0) + (size_t)p * a.K;
    }
}

// tile: LDS, element (r, c) at tile[r * TS + c]; scale: LDS [R]; t: tile index; NT: threads that share the
// tile (whole waves), tid: this thread's index among them; Ntot: total packed rows of the fused matrix.
template <int EPI, int TW, int NT>
__device__ __forceinline__ void epilogue_tile(const GemvArgs &a, const float *tile, int TS, const float *scale, int R,
                                              int t, int Ntot, int tid) {
    static_assert(TW >= 8 && TW <= 64 && (TW & (TW - 1)) == 0, "tile width");
    const int n_base = t * TW;
    if constexpr (EPI == EPI_PLAIN) {
        for (int idx = tid; idx < R * TW; idx += NT) {
            const int r = idx / TW, c = idx % TW;
            if (n_base + c < Ntot) a.y[(size_t)r * a.n0 + n_base + c] = tile[r * TS + c] * scale[r];
        }
    } else if constexpr (EPI == EPI_RESID) {
        const int total = ((R * TW + NT - 1) / NT) * NT;
        for (int idx = tid; idx < total; idx += NT) {
            const int r = idx / TW, c = idx % TW;
            const int n = n_base + c;
            float sq = 0.f;
            if (r < R && n < Ntot) {
                const size_t o = (size_t)r * a.n0 + n;
                const float gn = a.g_next != nullptr ? a.g_next[n] : 1.f;
                const float xn = a.xres[o] + tile[r * TS + c] * scale[r];
                a.xres[o] = xn;
                a.xg[o] = xn * gn;
                store_split_bf16(a.xgb, o, a.xgb_lo, xn * gn);
                sq = xn * xn;
            }
#pragma unroll
            for (int m = TW / 2; m >= 1; m >>= 1) sq += __shfl_xor(sq, m, WAVE);
            if (c == 0 && r < R) a.ssq_out[(size_t)r * a.ssq_stride + t] = sq;
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        constexpr int H2 = TW / 2;
        for (int idx = tid; idx < R * H2; idx += NT) {
            const int r = idx / H2, pj = idx % H2;
            const int j = t * H2 + pj;
            if (j < a.n0) {
                const float gt = tile[r * TS + pj] * scale[r];
                const float up = tile[r * TS + H2 + pj] * scale[r];
                const float v = gt / (1.f + __expf(-gt)) * up;
                const size_t o = (size_t)r * a.n0 + j;
                a.y[o] = v;
                store_split_bf16(a.yb, o, a.yb_lo, v);
            }
        }
    } else if constexpr (EPI == EPI_QKV) {
        constexpr int H2 = TW / 2;
        const int half = a.hd >> 1;
        for (int idx = tid; idx < R * H2; idx += NT) {
            const int r = idx / H2, pj = idx % H2;
            const int P = t * H2 + pj;
            if (P >= (Ntot >> 1)) continue;
            int hh = P / half;
            const int j = P % half;
            float y1 = tile[r * TS + pj] * scale[r];
            float y2 = tile[r * TS + H2 + pj] * scale[r];
            const int pos = a.row_pos[r];
            if (hh < a.nq + a.nkv) {
                const float c = a.rope_cos[(size_t)pos * half + j];
                const float s = a.rope_sin[(size_t)pos * half + j];
                const float r1 = y1 * c - y2 * s;
                const float r2 = y2 * c + y1 * s;
                y1 = r1; y2 = r2;
            }
            if (hh < a.nq) {
                const size_t o = (size_t)r * a.nq * a.hd + (size_t)hh * a.hd + j;
                a.y[o] = y1;
                a.y[o + half] = y2;
                store_split_bf16(a.yb, o, a.yb_lo, y1);
                store_split_bf16(a.yb, o + half, a.yb_lo, y2);
            } else {
                const bool is_k = hh < a.nq + a.nkv;
                const int kvh = hh - a.nq - (is_k ? 0 : a.nkv);
                const int seq = a.row_seq[r];
                kv_store(a.kv, a.kv_dtype, is_k, seq, pos, kvh, j, y1);
                kv_store(a.kv, a.kv_dtype, is_k, seq, pos, kvh, j + half, y2);
            }
        }
    } else if constexpr (EPI == EPI_LOGITS) {
        const int total = ((R * TW + NT - 1) / NT) * NT;
        for (int idx = tid; idx < total; idx += NT) {
            const int r = idx / TW, c = idx % TW;
            const int n = n_base + c;
            const bool valid = r < R && n < Ntot;
            const int rr = min(r, R - 1);
            const int orow = (a.y_rows != nullptr ? a.y_rows[rr] : rr) * a.y_mul + a.y_add;
            const float v = valid ? tile[rr * TS + c] * scale[rr] : -INFINITY;
            if (valid) a.y[(size_t)orow * a.y_stride + n] = v;
            float m = v;
            int arg = valid ? n : 0x7fffffff;
#pragma unroll
            for (int msk = TW / 2; msk >= 1; msk >>= 1) {
                const float om = __shfl_xor(m, msk, WAVE);
                const int oa = __shfl_xor(arg, msk, WAVE);
                if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
            }
            double e = valid ? exp((double)(v - m) * (double)a.inv_t) : 0.0;
#pragma unroll
            for (int msk = TW / 2; msk >= 1; msk >>= 1) e += __shfl_xor(e, msk, WAVE);
            if (c == 0 && r < R) {
                const size_t pi = (size_t)orow * a.n_tiles + t;
                a.pm[pi] = m;
                a.ps[pi] = e;
                a.pa[pi] = arg;
            }
        }
    }
}

// Operands of a residual / QKV epilogue that do not depend on the projection's result, fetched by the
// persistent kernel before the matrix instructions of the group so that the epilogue itself is free of loads.
// One thread per output element of a 16-column tile (residual: R x 16, QKV: R x 8 pairs).
struct EpiPre {
    float xres, gn;        // RESID: residual element, weight of the next norm
    float cs, sn;          // QKV: rotary cosine / sine of this row's position and this pair's frequency
    int pos, seq, page;    // QKV: row position, sequence, physical KV page (fetched once per kernel)
};

template <int EPI>
__device__ __forceinline__ void epi_prefetch_rows(const GemvArgs &a, int R, int tid, EpiPre &p) {
    if constexpr (EPI == EPI_QKV) {
        const int r = tid >> 3;
        p.pos = 0; p.seq = 0; p.page = 0;
        if (r < R) {
            p.pos = a.row_pos[r];
            p.seq = a.row_seq[r];
            p.page = kv_page(a.kv, p.seq, p.pos);
        }
    }
}

template <int EPI>
__device__ __forceinline__ void epi_prefetch_group(const GemvArgs &a, int R, int t, int Ntot, int tid, EpiPre &p) {
    if constexpr (EPI == EPI_RESID) {
        const int r = tid >> 4, n = t * 16 + (tid & 15);
        p.xres = 0.f; p.gn = 1.f;
        if (r < R && n < Ntot) {
            p.xres = a.xres[(size_t)r * a.n0 + n];
            if (a.g_next != nullptr) p.gn = a.g_next[n];
        }
    } else if constexpr (EPI == EPI_QKV) {
        const int r = tid >> 3, half = a.hd >> 1;
        const int P = t * 8 + (tid & 7);
        p.cs = 1.f; p.sn = 0.f;
        if (r < R && P < (Ntot >> 1) && P / half < a.nq + a.nkv) {
            p.cs = a.rope_cos[(size_t)p.pos * half + P % half];
            p.sn = a.rope_sin[(size_t)p.pos * half + P % half];
        }
    }
}

// The residual and QKV epilogues of epilogue_tile for a 16-column tile and at least 16 R threads, on prefetched
// operands: the same arithmetic in the same order.
template <int EPI>
__device__ __forceinline__ void epilogue_tile_pre(const GemvArgs &a, const float *tile, int TS, const float *scale, int R,
                                                  int t, int Ntot, int tid, const EpiPre &p) {
    if constexpr (EPI == EPI_RESID) {
        if (tid >= ((R * 16 + 63) & ~63)) return;  // whole waves: the shuffles below need their 16-lane groups
        const int r = tid >> 4, c = tid & 15;
        const int n = t * 16 + c;
        float sq = 0.f;
        if (r < R && n < Ntot) {
            const size_t o = (size_t)r * a.n0 + n;
            const float xn = p.xres + tile[r * TS + c] * scale[r];
            a.xres[o] = xn;
            a.xg[o] = xn * p.gn;
            store_split_bf16(a.xgb, o, a.xgb_lo, xn * p.gn);
            sq = xn * xn;
        }
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) sq += __shfl_xor(sq, m, WAVE);
        if (c == 0 && r < R) a.ssq_out[(size_t)r * a.ssq_stride + t] = sq;
    } else if constexpr (EPI == EPI_QKV) {
        const int r = tid >> 3, pj = tid & 7;
        if (r >= R) return;
        const int half = a.hd >> 1;
        const int P = t * 8 + pj;
        if (P >= (Ntot >> 1)) return;
        int hh = P / half;
        const int j = P % half;
        float y1 = tile[r * TS + pj] * scale[r];
        float y2 = tile[r * TS + 8 + pj] * scale[r];
        if (hh < a.nq + a.nkv) {
            const float r1 = y1 * p.cs - y2 * p.sn;
            const float r2 = y2 * p.cs + y1 * p.sn;
            y1 = r1; y2 = r2;
        }
        if (hh < a.nq) {
            const size_t o = (size_t)r * a.nq * a.hd + (size_t)hh * a.hd + j;
            a.y[o] = y1;
            a.y[o + half] = y2;
            store_split_bf16(a.yb, o, a.yb_lo, y1);
            store_split_bf16(a.yb, o + half, a.yb_lo, y2);
        } else {
            const bool is_k = hh < a.nq + a.nkv;
            const int kvh = hh - a.nq - (is_k ? 0 : a.nkv);
            const int in_page = p.pos & (a.kv.page_tokens - 1);
            const size_t base = kv_head_base(a.kv, p.page, kvh);
            const size_t e1 = base + (is_k ? kv_in_k(a.kv, in_page, j) : kv_in_v(a.kv, in_page, j));
            const size_t e2 = base + (is_k ? kv_in_k(a.kv, in_page, j + half) : kv_in_v(a.kv, in_page, j + half));
            void *pool = is_k ? a.kv.k : a.kv.v;
            if (a.kv_dtype == DT_BF16) {
                reinterpret_cast<bf16_t *>(pool)[e1] = f32_to_bf16(y1);
                reinterpret_cast<bf16_t *>(pool)[e2] = f32_to_bf16(y2);
            } else {
                reinterpret_cast<float *>(pool)[e1] = y1;
                reinterpret_cast<float *>(pool)[e2] = y2;
            }
        }
    }
}

// Row scales rsqrt(mean(x^2) + eps) from the sum-of-squares slots of the producer (1 when the input is
// not normed).  One wave per row, lanes over slots.  The slot loads are issued by begin() before the
// weight stream starts and consumed by finish() after it, so their latency is hidden; shapes that do not
// fit the register budget (more than SC_ROWS rows per wave or more than 64 * SC_REGS slots) load late.
constexpr int SC_ROWS = 5;
constexpr int SC_REGS = 4;

template <int NT, int ROWS = SC_ROWS>
struct RowScales {
    float v[ROWS][SC_REGS];
    bool early;

    __device__ __forceinline__ void begin(const GemvArgs &a, int R) {
        constexpr int NW = NT / 64;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        early = a.ssq_in != nullptr && R <= NW * ROWS && a.ssq_in_slots <= 64 * SC_REGS;
        if (!early) return;
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int r = wave + NW * i;
            const int xr = min(r, R - 1) * a.x_mul + a.x_add;
#pragma unroll
            for (int q = 0; q < SC_REGS; ++q) {
                const int slot = lane + 64 * q;
                v[i][q] = (r < R && slot < a.ssq_in_slots) ? a.ssq_in[(size_t)xr * a.ssq_stride + slot] : 0.f;
            }
        }
    }

    // writes scale[0..R) in LDS and ends with a barrier
    __device__ __forceinline__ void finish(const GemvArgs &a, float *scale, int R) {
        constexpr int NW = NT / 64;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        if (a.ssq_in == nullptr) {
            for (int r = threadIdx.x; r < R; r += NT) scale[r] = 1.f;
        } else if (early) {
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                const int r = wave + NW * i;
                float s = 0.f;
#pragma unroll
                for (int q = 0; q < SC_REGS; ++q) s += v[i][q];
                s = wave_sum(s);
                if (lane == 0 && r < R) scale[r] = rsqrtf(s / (float)a.K + a.eps);
            }
        } else {
            for (int r = wave; r < R; r += NW) {
                const int xr = r * a.x_mul + a.x_add;
                float s = 0.f;
                for (int slot = lane; slot < a.ssq_in_slots; slot += 64) s += a.ssq_in[(size_t)xr * a.ssq_stride + slot];
                s = wave_sum(s);
                if (lane == 0) scale[r] = rsqrtf(s / (float)a.K + a.eps);
            }
        }
        __syncthreads();
    }
};

}  // namespace sd
