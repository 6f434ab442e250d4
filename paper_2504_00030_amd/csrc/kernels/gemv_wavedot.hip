// Weight-streaming projections for few rows (draft decode, small gamma, fp32 models):
// every wave owns a few weight rows, the 64 lanes split K with 16-byte loads, partial dot
// products are reduced across the wave, and the epilogue (RoPE + KV write, residual add with
// the statistics of the next RMSNorm, SwiGLU, logits with softmax partials) runs in the same
// kernel.  No LDS on the streaming path; the x rows are re-read from L1/L2.
//
// This is the draft model's decode step and the small-gamma verify pass of a speculative
// step (Background section: T_draft per drafted token, T_target per verification).
#include "common.hpp"
#include "epilogue.hpp"
#include "kv.hpp"
#include "params.hpp"

namespace sd {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Weights are read once per launch: non-temporal loads keep them from evicting x and the KV cache.
template <typename WT> struct WVec;
template <> struct WVec<float> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ void load(const float *p, float (&o)[4]) {
        const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
};
template <> struct WVec<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ void load(const bf16_t *p, float (&o)[8]) {
        const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
        o[0] = bf16_lo(v.x); o[1] = bf16_hi(v.x); o[2] = bf16_lo(v.y); o[3] = bf16_hi(v.y);
        o[4] = bf16_lo(v.z); o[5] = bf16_hi(v.z); o[6] = bf16_lo(v.w); o[7] = bf16_hi(v.w);
    }
};

constexpr int SLOT_REGS = 8;  // up to 512 sum-of-squares slots per row

__device__ __forceinline__ int total_rows(const GemvArgs &a, int epi) {
    if (epi == EPI_QKV) return (a.nq + 2 * a.nkv) * a.hd;
    if (epi == EPI_SWIGLU) return 2 * a.n0;
    return a.n0;
}

// Weight row behind wave-row index t (see the launcher for the index spaces).
template <typename WT, int EPI, int NR>
__device__ __forceinline__ const WT *wrow(const GemvArgs &a, int t) {
    if constexpr (EPI == EPI_SWIGLU) {
        const int gi = t / NR, pos = t % NR;
        const int j = gi * (NR / 2) + pos % (NR / 2);
        const WT *base = reinterpret_cast<const WT *>(pos < NR / 2 ? a.w0 : a.w1);
        return base + (size_t)j * a.K;
    } else if constexpr (EPI == EPI_QKV) {
        const int half = a.hd >> 1;
        const int gi = t / NR, pos = t % NR;
        const int P = gi * (NR / 2) + pos % (NR / 2);
        int hh = P / half;
        const int j = P % half + (pos < NR / 2 ? 0 : half);
        const WT *base;
        if (hh < a.nq) base = reinterpret_cast<const WT *>(a.w0);
        else if (hh < a.nq + a.nkv) { base = reinterpret_cast<const WT *>(a.w1); hh -= a.nq; }
        else { base = reinterpret_cast<const WT *>(a.w2); hh -= a.nq + a.nkv; }
        return base + ((size_t)hh * a.hd + j) * a.K;
    } else {
        return reinterpret_cast<const WT *>(a.w0) + (size_t)t * a.K;
    }
}

template <typename WT, int RC, int EPI, int NR>
__global__ __launch_bounds__(256) void gemv_wavedot_k(const GemvArgs a) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int VEC = WVec<WT>::VEC;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wid = blockIdx.x * 4 + wave;
    const int Ntot = total_rows(a, EPI);
    const int t_begin = wid * a.rpw;
    const int K = a.K;
    __shared__ float lds_ssq[4][128];
    __shared__ float lds_m[4][4];
    __shared__ double lds_e[4][4];
    __shared__ int lds_a[4][4];

    for (int r0 = 0; r0 < a.R; r0 += RC) {
        // input rows of this chunk (clamped: a surplus row repeats the last one and is not written)
        const float *xr[RC];
        int xrow[RC];
#pragma unroll
        for (int rc = 0; rc < RC; ++rc) {
            const int r = min(r0 + rc, a.R - 1);
            xrow[rc] = r * a.x_mul + a.x_add;
            xr[rc] = a.x + (size_t)xrow[rc] * K;
        }
        // partial sums of squares of the input rows: issued now, reduced after the streaming loop
        float sl[RC][SLOT_REGS];
        if (a.ssq_in != nullptr) {
#pragma unroll
            for (int rc = 0; rc < RC; ++rc)
#pragma unroll
                for (int i = 0; i < SLOT_REGS; ++i) {
                    const int s = lane + i * 64;
                    sl[rc][i] = s < a.ssq_in_slots ? a.ssq_in[(size_t)xrow[rc] * a.ssq_stride + s] : 0.f;
                }
        }
        float scale[RC];
#pragma unroll
        for (int rc = 0; rc < RC; ++rc) scale[rc] = 1.f;
        bool scale_done = false;

        float ssq_acc[RC];
#pragma unroll
        for (int rc = 0; rc < RC; ++rc) ssq_acc[rc] = 0.f;
        float mine = -INFINITY;  // LOGITS: the logit this lane keeps

        for (int g = 0; g < a.rpw; g += NR) {
            const int t0 = t_begin + g;
            if (t0 >= Ntot) break;
            const WT *wp[NR];
#pragma unroll
            for (int nr = 0; nr < NR; ++nr) wp[nr] = wrow<WT, EPI, NR>(a, min(t0 + nr, Ntot - 1));
            float acc[NR][RC];
#pragma unroll
            for (int nr = 0; nr < NR; ++nr)
#pragma unroll
                for (int rc = 0; rc < RC; ++rc) acc[nr][rc] = 0.f;

#pragma unroll 2
            for (int k = lane * VEC; k < K; k += 64 * VEC) {
                float wv[NR][VEC];
#pragma unroll
                for (int nr = 0; nr < NR; ++nr) WVec<WT>::load(wp[nr] + k, wv[nr]);
#pragma unroll
                for (int rc = 0; rc < RC; ++rc) {
                    float xv[VEC];
#pragma unroll
                    for (int q = 0; q < VEC / 4; ++q) {
                        const float4 v = *reinterpret_cast<const float4 *>(xr[rc] + k + 4 * q);
                        xv[4 * q] = v.x; xv[4 * q + 1] = v.y; xv[4 * q + 2] = v.z; xv[4 * q + 3] = v.w;
                    }
#pragma unroll
                    for (int nr = 0; nr < NR; ++nr)
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[nr][rc] = fmaf(wv[nr][e], xv[e], acc[nr][rc]);
                }
            }
#pragma unroll
            for (int nr = 0; nr < NR; ++nr)
#pragma unroll
                for (int rc = 0; rc < RC; ++rc) acc[nr][rc] = wave_sum(acc[nr][rc]);

            if (a.ssq_in != nullptr && !scale_done) {
#pragma unroll
                for (int rc = 0; rc < RC; ++rc) {
                    float s = 0.f;
#pragma unroll
                    for (int i = 0; i < SLOT_REGS; ++i) s += sl[rc][i];
                    s = wave_sum(s);
                    scale[rc] = rsqrtf(s / (float)K + a.eps);
                }
                scale_done = true;
            }

            // ---------------- epilogue of this group: values are uniform across the wave ----------------
            if constexpr (EPI == EPI_PLAIN) {
#pragma unroll
                for (int nr = 0; nr < NR; ++nr)
#pragma unroll
                    for (int rc = 0; rc < RC; ++rc)
                        if (lane == nr * RC + rc && t0 + nr < Ntot && r0 + rc < a.R)
                            a.y[(size_t)(r0 + rc) * a.n0 + t0 + nr] = acc[nr][rc] * scale[rc];
            } else if constexpr (EPI == EPI_RESID) {
#pragma unroll
                for (int nr = 0; nr < NR; ++nr) {
                    const int n = t0 + nr;
                    if (n >= Ntot) continue;
                    const float gn = a.g_next != nullptr ? a.g_next[n] : 1.f;
#pragma unroll
                    for (int rc = 0; rc < RC; ++rc) {
                        if (r0 + rc >= a.R) continue;
                        const size_t o = (size_t)(r0 + rc) * a.n0 + n;
                        const float xn = a.xres[o] + acc[nr][rc] * scale[rc];
                        ssq_acc[rc] += xn * xn;
                        if (lane == 0) {
                            a.xres[o] = xn;
                            a.xg[o] = xn * gn;
                            a.xgb[o] = f32_to_bf16(xn * gn);
                        }
                    }
                }
            } else if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int pi = 0; pi < NR / 2; ++pi)
#pragma unroll
                    for (int rc = 0; rc < RC; ++rc)
                        if (lane == pi * RC + rc && r0 + rc < a.R) {
                            const int j = (t0 / NR) * (NR / 2) + pi;
                            const float gt = acc[pi][rc] * scale[rc];
                            const float up = acc[pi + NR / 2][rc] * scale[rc];
                            const float v = gt / (1.f + __expf(-gt)) * up;
                            const size_t o = (size_t)(r0 + rc) * a.n0 + j;
                            a.y[o] = v;
                            a.yb[o] = f32_to_bf16(v);
                        }
            } else if constexpr (EPI == EPI_QKV) {
                const int half = a.hd >> 1;
#pragma unroll
                for (int pi = 0; pi < NR / 2; ++pi)
#pragma unroll
                    for (int rc = 0; rc < RC; ++rc)
                        if (lane == pi * RC + rc && r0 + rc < a.R) {
                            const int r = r0 + rc;
                            const int P = (t0 / NR) * (NR / 2) + pi;
                            int hh = P / half;
                            const int j = P % half;
                            float y1 = acc[pi][rc] * scale[rc];
                            float y2 = acc[pi + NR / 2][rc] * scale[rc];
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
#pragma unroll
                for (int nr = 0; nr < NR; ++nr)
#pragma unroll
                    for (int rc = 0; rc < RC; ++rc)
                        if (lane == (g + nr) * RC + rc) mine = acc[nr][rc] * scale[rc];
            }
        }

        if constexpr (EPI == EPI_RESID) {
#pragma unroll
            for (int rc = 0; rc < RC; ++rc)
                if (lane == 0 && r0 + rc < a.R) lds_ssq[wave][r0 + rc] = ssq_acc[rc];
        }
        if constexpr (EPI == EPI_LOGITS) {
            // lane = local_row * RC + rc holds one logit; reduce over the lanes with the same rc
            const int rc = lane % RC;
            const int n = t_begin + lane / RC;
            const int r = r0 + rc;
            const bool valid = lane < a.rpw * RC && n < Ntot && r < a.R && t_begin < Ntot;
            const int lrow = min(r, a.R - 1);
            const int orow = (a.y_rows != nullptr ? a.y_rows[lrow] : lrow) * a.y_mul + a.y_add;
            float v = valid ? mine : -INFINITY;
            if (valid) a.y[(size_t)orow * a.y_stride + n] = v;
            float m = v;
            int arg = valid ? n : 0x7fffffff;
#pragma unroll
            for (int msk = RC; msk < 64; msk <<= 1) {
                const float om = __shfl_xor(m, msk, WAVE);
                const int oa = __shfl_xor(arg, msk, WAVE);
                if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
            }
            double e = valid ? exp((double)(v - m) * (double)a.inv_t) : 0.0;
#pragma unroll
            for (int msk = RC; msk < 64; msk <<= 1) e += __shfl_xor(e, msk, WAVE);
            // merge the four waves of the workgroup: one partial per (row, workgroup), in wave order
            if (lane < RC) {
                lds_m[wave][lane] = m;
                lds_e[wave][lane] = e;
                lds_a[wave][lane] = arg;
            }
            __syncthreads();
            if (wave == 0 && lane < RC && r < a.R) {
                float M = lds_m[0][lane];
                int A = lds_a[0][lane];
#pragma unroll
                for (int w = 1; w < 4; ++w)
                    if (lds_m[w][lane] > M || (lds_m[w][lane] == M && lds_a[w][lane] < A)) {
                        M = lds_m[w][lane];
                        A = lds_a[w][lane];
                    }
                double S = 0.0;
#pragma unroll
                for (int w = 0; w < 4; ++w)
                    if (lds_m[w][lane] != -INFINITY)
                        S += lds_e[w][lane] * exp((double)(lds_m[w][lane] - M) * (double)a.inv_t);
                const size_t pi = (size_t)orow * a.n_tiles + blockIdx.x;
                a.pm[pi] = M;
                a.ps[pi] = S;
                a.pa[pi] = A;
            }
            __syncthreads();
        }
    }

    if constexpr (EPI == EPI_RESID) {
        // one slot per workgroup (a wave that owns no rows has written zeros)
        __syncthreads();
        for (int r = threadIdx.x; r < a.R; r += 256)
            a.ssq_out[(size_t)r * a.ssq_stride + blockIdx.x] =
                lds_ssq[0][r] + lds_ssq[1][r] + lds_ssq[2][r] + lds_ssq[3][r];
    }
}

// ---- split-K variant for one or two rows (draft decode) ---------------------------------------------
// A workgroup of NW waves owns TW packed weight rows.  The waves form KS k-slices x (NW / KS) row
// slots; a wave keeps its slice of the x rows in registers (read once), streams its slice of each of
// its weight rows with one 16-byte load per lane and step, and leaves one partial dot product per
// (row, slice) in LDS.  The slices are summed in slice order and the shared tile epilogue runs.
constexpr int WS_MAX_WGS = 512;
constexpr int WS_STEPS = 4;  // k-steps (of 64 lanes x 16 bytes) a wave can hold of each x row

template <typename WT, int RC, int EPI, int TW, int NW>
__global__ __launch_bounds__(NW * 64) void gemv_wsplit_k(const GemvArgs a, const int KS, const int n_tiles_total) {
    if (a.active != nullptr && *a.active == 0) return;
    constexpr int NT = NW * 64;
    constexpr int VEC = WVec<WT>::VEC;
    constexpr int STEP = 64 * VEC;
    constexpr int NR = TW >= 16 ? 8 : 4;  // rows streamed together by a wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int Ntot = total_rows(a, EPI);
    const int K = a.K;
    const int RS = NW / KS;              // row slots
    const int wk = wave % KS, wr = wave / KS;
    const int RPS = TW / RS;             // rows per slot (host guarantees TW % RS == 0)
    const int steps = (K + STEP - 1) / STEP;
    const int SPS = (steps + KS - 1) / KS;  // steps per slice, <= WS_STEPS
    const int k0 = wk * SPS * STEP + lane * VEC;

    __shared__ float part[TW * NW * RC];   // [row][slice][rc], slices < KS used
    __shared__ float tile[RC * (TW + 1)];
    __shared__ float s_scale[RC];

    RowScales<NT> rs;
    rs.begin(a, RC);

    // this wave's slice of the x rows
    float xs[RC][WS_STEPS][VEC];
#pragma unroll
    for (int rc = 0; rc < RC; ++rc) {
        const float *xr = a.x + (size_t)(rc * a.x_mul + a.x_add) * K;
#pragma unroll
        for (int st = 0; st < WS_STEPS; ++st) {
            const int k = k0 + st * STEP;
            const bool in = st < SPS && k < K;
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
                const float4 v = in ? *reinterpret_cast<const float4 *>(xr + k + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
                xs[rc][st][4 * q] = v.x; xs[rc][st][4 * q + 1] = v.y; xs[rc][st][4 * q + 2] = v.z; xs[rc][st][4 * q + 3] = v.w;
            }
        }
    }

  // a workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ...; its x slices stay in registers
  for (int t = blockIdx.x; t < n_tiles_total; t += gridDim.x) {
    const int p_base = t * TW + wr * RPS;
    for (int lr0 = 0; lr0 < RPS; lr0 += NR) {
        const WT *wp[NR];
#pragma unroll
        for (int nr = 0; nr < NR; ++nr) wp[nr] = packed_row<WT, EPI>(a, min(p_base + min(lr0 + nr, RPS - 1), Ntot - 1), TW);
        float acc[NR][RC];
#pragma unroll
        for (int nr = 0; nr < NR; ++nr)
#pragma unroll
            for (int rc = 0; rc < RC; ++rc) acc[nr][rc] = 0.f;
#pragma unroll
        for (int st = 0; st < WS_STEPS; ++st) {
            const int k = k0 + st * STEP;
            if (st < SPS && k < K) {
                float wv[NR][VEC];
#pragma unroll
                for (int nr = 0; nr < NR; ++nr) WVec<WT>::load(wp[nr] + k, wv[nr]);
#pragma unroll
                for (int nr = 0; nr < NR; ++nr)
#pragma unroll
                    for (int rc = 0; rc < RC; ++rc)
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[nr][rc] = fmaf(wv[nr][e], xs[rc][st][e], acc[nr][rc]);
            }
        }
#pragma unroll
        for (int nr = 0; nr < NR; ++nr)
#pragma unroll
            for (int rc = 0; rc < RC; ++rc) {
                const float v = wave_sum(acc[nr][rc]);
                if (lane == 0 && lr0 + nr < RPS) part[((wr * RPS + lr0 + nr) * NW + wk) * RC + rc] = v;
            }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < TW * RC; idx += NT) {
        const int row = idx / RC, rc = idx % RC;
        float s = 0.f;
        for (int w = 0; w < KS; ++w) s += part[(row * NW + w) * RC + rc];
        tile[rc * (TW + 1) + row] = s;
    }
    if (t == (int)blockIdx.x) rs.finish(a, s_scale, RC);  // ends with a barrier
    else __syncthreads();
    epilogue_tile<EPI, TW, NT>(a, tile, TW + 1, s_scale, RC, t, Ntot, threadIdx.x);
    __syncthreads();  // part / tile are reused by the next tile
  }
}

struct WsplitCfg { int tw, ks; bool ok; };

// Tile width and k-slices for the split-K kernel (NW = 8 waves), or ok = false when the shape does not fit.
static WsplitCfg wsplit_cfg(int epi, int Ntot, int K, int R, int w_dtype) {
    WsplitCfg c{16, 8, false};
    if (R > 2) return c;
    const int step = 64 * (w_dtype == DT_BF16 ? 8 : 4);
    const int steps = (K + step - 1) / step;
    int ks = 8;
    while (ks > 1 && ks > steps) ks >>= 1;     // never more slices than steps
    if ((steps + ks - 1) / ks > WS_STEPS) return c;
    int tw = 16;
    if (epi == EPI_LOGITS) tw = 64;
    else if (Ntot / 16 < 256) tw = 8;
    const int rs = 8 / ks;
    if (tw < rs) tw = rs < 8 ? 8 : rs;
    if (tw % rs) return c;
    c.tw = tw; c.ks = ks; c.ok = true;
    return c;
}

bool gemv_wavedot_uses_split(int epi, int Ntot, int K, int R, int w_dtype) {
    return wsplit_cfg(epi, Ntot, K, R, w_dtype).ok;
}

int gemv_wavedot_tile_cols(int epi, int Ntot, int K, int R, int w_dtype) {
    const WsplitCfg c = wsplit_cfg(epi, Ntot, K, R, w_dtype);
    if (c.ok) return c.tw;
    return 4 * gemv_wavedot_pick_rpw(epi, Ntot, K, R, w_dtype);
}

template <typename WT, int RC, int EPI>
static hipError_t launch_wsplit(const GemvArgs &a, int Ntot, const WsplitCfg &c, hipStream_t s) {
    const int tiles = (Ntot + c.tw - 1) / c.tw;
    // at most WS_MAX_WGS workgroups (two per CU): beyond that a workgroup loops over several tiles
    const int blocks = tiles < WS_MAX_WGS ? tiles : WS_MAX_WGS;
    if (c.tw == 8) hipLaunchKernelGGL((gemv_wsplit_k<WT, RC, EPI, 8, 8>), dim3(blocks), dim3(512), 0, s, a, c.ks, tiles);
    else if (c.tw == 16) hipLaunchKernelGGL((gemv_wsplit_k<WT, RC, EPI, 16, 8>), dim3(blocks), dim3(512), 0, s, a, c.ks, tiles);
    else hipLaunchKernelGGL((gemv_wsplit_k<WT, RC, EPI, 64, 8>), dim3(blocks), dim3(512), 0, s, a, c.ks, tiles);
    return hipGetLastError();
}

// rows per wave: enough waves to fill the chip, long enough streams per wave
int gemv_wavedot_pick_rpw(int epi, int Ntot, int K, int R, int w_dtype) {
    (void)K; (void)w_dtype;
    const int RC = R == 1 ? 1 : (R == 2 ? 2 : 4);
    if (epi == EPI_LOGITS) return 64 / RC;
    if (Ntot / 4 < 1024) return 2;     // NR = 2 variant
    int rpw = (Ntot / 4096) & ~3;
    if (rpw < 4) rpw = 4;
    if (rpw > 16) rpw = 16;
    return rpw;
}

template <typename WT, int RC, int EPI>
static hipError_t launch_nr(const GemvArgs &a, int Ntot, hipStream_t s) {
    const int waves = (Ntot + a.rpw - 1) / a.rpw;
    const int blocks = (waves + 3) / 4;
    if (a.rpw % 4 == 0)
        hipLaunchKernelGGL((gemv_wavedot_k<WT, RC, EPI, 4>), dim3(blocks), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL((gemv_wavedot_k<WT, RC, EPI, 2>), dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <typename WT, int EPI>
static hipError_t launch_rc(const GemvArgs &a, int Ntot, hipStream_t s) {
    const WsplitCfg c = wsplit_cfg(EPI, Ntot, a.K, a.R, sizeof(WT) == 2 ? DT_BF16 : DT_F32);
    if (c.ok && a.rpw == 0) {
        if (a.R == 1) return launch_wsplit<WT, 1, EPI>(a, Ntot, c, s);
        return launch_wsplit<WT, 2, EPI>(a, Ntot, c, s);
    }
    if (a.R == 1) return launch_nr<WT, 1, EPI>(a, Ntot, s);
    if (a.R == 2) return launch_nr<WT, 2, EPI>(a, Ntot, s);
    return launch_nr<WT, 4, EPI>(a, Ntot, s);
}

template <typename WT>
static hipError_t launch_epi(const GemvArgs &a, int epi, hipStream_t s) {
    int Ntot = a.n0;
    if (epi == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (epi == EPI_SWIGLU) Ntot = 2 * a.n0;
    switch (epi) {
        case EPI_PLAIN: return launch_rc<WT, EPI_PLAIN>(a, Ntot, s);
        case EPI_QKV: return launch_rc<WT, EPI_QKV>(a, Ntot, s);
        case EPI_RESID: return launch_rc<WT, EPI_RESID>(a, Ntot, s);
        case EPI_SWIGLU: return launch_rc<WT, EPI_SWIGLU>(a, Ntot, s);
        case EPI_LOGITS: return launch_rc<WT, EPI_LOGITS>(a, Ntot, s);
    }
    return hipErrorInvalidValue;
}

// Host-side contract (checked by the engine before the first launch):
//   K % VEC == 0, rows 16-byte aligned, rpw even, rpw % 4 == 0 or rpw == 2,
//   SWIGLU: n0 % (NR/2) == 0; QKV: (hd/2) % (NR/2) == 0; LOGITS: rpw * RC <= 64;
//   RESID: R <= 128, gridDim.x <= ssq_stride; ssq_in_slots <= 512.
// rpw == 0 selects the split-K kernel (shapes for which gemv_wavedot_uses_split() is true).
hipError_t launch_gemv_wavedot(const GemvArgs &a, int epi, int w_dtype, hipStream_t s) {
    if (a.R < 1 || (a.rpw != 0 && a.rpw < 2)) return hipErrorInvalidValue;
    if (a.rpw == 0 && !gemv_wavedot_uses_split(epi, epi == EPI_QKV ? (a.nq + 2 * a.nkv) * a.hd : (epi == EPI_SWIGLU ? 2 * a.n0 : a.n0),
                                               a.K, a.R, w_dtype))
        return hipErrorInvalidValue;
    if (w_dtype == DT_BF16) return launch_epi<bf16_t>(a, epi, s);
    return launch_epi<float>(a, epi, s);
}

}  // namespace sd
