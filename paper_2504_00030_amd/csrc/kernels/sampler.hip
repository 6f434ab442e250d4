// Sampling side of a speculative step (Background section; accept / resample rule of the
// speculative-sampling works cited there):
//   draft_sample_k   x_i ~ softmax(draft logits / T) by index-order inverse CDF (argmax if T == 0),
//                    the draft's confidence for GammaTune+ early stopping
//   accept_scan_k    softmax normalisers of the target rows, the test u * q(x) < p(x) row by row,
//                    the bonus draw when every drafted token is accepted
//   residual_k       draw from norm(max(0, p - q)) at the first refused row, then commit the step
// The logits kernels leave per-tile (max, sum exp, argmax) partials, so the normalisers cost one
// pass over a few hundred numbers per row; only the refused row is swept in full.  All sampling
// arithmetic is fp64; every reduction has a fixed order, so results repeat bit for bit.
#include "common.hpp"
#include "params.hpp"

namespace sd {

__device__ __forceinline__ double wave_scan_incl(double v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const double o = __shfl_up(v, d, WAVE);
        if (lane >= d) v += o;
    }
    return v;
}

struct RowStats {
    double M, S;
    int arg;
};

// Softmax partials of one logits row on two levels: level 1 has one (max, sum exp, argmax) per tile of
// `tile` vocabulary entries (left by the logits kernel), level 2 one per 64 consecutive level-1 tiles
// (left by merge_partials_k).
struct PartRow {
    const float *pm1; const double *ps1; const int32_t *pa1; int n1, tile;
    const float *pm2; const double *ps2; const int32_t *pa2; int n2;
};

__device__ __forceinline__ PartRow part_row(const float *pm, const double *ps, const int32_t *pa, int n1, int tile,
                                            const float *pm2, const double *ps2, const int32_t *pa2, int n2, size_t row) {
    PartRow p;
    p.pm1 = pm + row * n1; p.ps1 = ps + row * n1; p.pa1 = pa + row * n1; p.n1 = n1; p.tile = tile;
    p.pm2 = pm2 + row * n2; p.ps2 = ps2 + row * n2; p.pa2 = pa2 + row * n2; p.n2 = n2;
    return p;
}

// One wave reduces n partials (max with lowest-index argmax, then sum of rescaled sums).
__device__ RowStats wave_reduce_partials(const float *pm, const double *ps, const int32_t *pa, int n, double inv_t,
                                         int lane) {
    float m = -INFINITY;
    int arg = 0x7fffffff;
    for (int t = lane; t < n; t += 64) {
        const float v = pm[t];
        const int ai = pa[t];
        if (v > m || (v == m && ai < arg)) { m = v; arg = ai; }
    }
#pragma unroll
    for (int msk = 32; msk >= 1; msk >>= 1) {
        const float om = __shfl_xor(m, msk, WAVE);
        const int oa = __shfl_xor(arg, msk, WAVE);
        if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
    }
    double s = 0.0;
    for (int t = lane; t < n; t += 64) s += ps[t] * exp((double)(pm[t] - m) * inv_t);
    s = wave_sum(s);
    RowStats r;
    r.M = (double)m; r.S = s; r.arg = arg;  // arg stays 0x7fffffff when no entry compares (empty or all-NaN input)
    return r;
}

// Statistics of one logits row from its level-2 partials, computed by one wave.
__device__ __forceinline__ RowStats wave_row_stats(const PartRow &p, double inv_t, int lane) {
    return wave_reduce_partials(p.pm2, p.ps2, p.pa2, p.n2, inv_t, lane);
}

// First index i in [0, n) whose inclusive running sum base + c_0 + .. + c_i exceeds target, where
// c_i = ps[i] * exp((pm[i] - M) * inv_t); lanes own contiguous runs so the order is index order.
// Returns the index (or n - 1 when rounding leaves no crossing) and the running sum before it.
__device__ __forceinline__ int wave_find_partial(const float *pm, const double *ps, int n, double M, double inv_t,
                                                 double base, double target, int lane, double *before) {
    const int per = (n + 63) / 64;
    const int b0 = lane * per, b1 = min(b0 + per, n);
    double seg = 0.0;
    for (int i = b0; i < b1; ++i) seg += ps[i] * exp(((double)pm[i] - M) * inv_t);
    const double incl = base + wave_scan_incl(seg, lane);
    const unsigned long long hit = __ballot(incl > target && b0 < b1);
    int idx = n - 1;
    double bef = 0.0;
    if (hit) {
        const int src = __ffsll((long long)hit) - 1;
        double cum = incl - seg;
        int is = b1 - 1;
        double ib = cum;
        bool f = false;
        for (int i = b0; i < b1; ++i) {
            const double c = ps[i] * exp(((double)pm[i] - M) * inv_t);
            if (!f) {
                ib = cum;  // stays at "before the last entry of the run" when rounding hides the crossing
                if (cum + c > target) { is = i; f = true; }
            }
            cum += c;
        }
        idx = __shfl(is, src, WAVE);
        bef = __shfl(ib, src, WAVE);
    } else {
        // running sum before the last entry
        const double tot = __shfl(incl, 63, WAVE);
        bef = tot - ps[n - 1] * exp(((double)pm[n - 1] - M) * inv_t);
    }
    *before = bef;
    return idx;
}

// Index-order inverse CDF over one row, by one wave: first j with cum_j > target, where the weights are
// w_j = exp((l_j - M) * inv_t).  The crossing is located on level 2, then among the 64 level-1 tiles
// below it, then element by element inside that tile.  If rounding leaves no crossing the last index
// of the innermost range is returned.
__device__ int wave_sample_row(const float *logits, int vocab, const PartRow &p, double M, double inv_t, double target,
                               int lane) {
    double base2 = 0.0;
    const int j2 = wave_find_partial(p.pm2, p.ps2, p.n2, M, inv_t, 0.0, target, lane, &base2);
    const int t_lo = j2 * 64, t_n = min(64, p.n1 - t_lo);
    double base1 = 0.0;
    const int t_star = t_lo + wave_find_partial(p.pm1 + t_lo, p.ps1 + t_lo, t_n, M, inv_t, base2, target, lane, &base1);
    // inside the tile: contiguous elements per lane
    const int e0 = t_star * p.tile;
    const int len = min(p.tile, vocab - e0);
    const int epl = (len + 63) / 64;
    const int eb = lane * epl, ee = min(eb + epl, len);
    double w[8];
    double sseg = 0.0;
    for (int i = 0; i < 8; ++i) {
        const int e = eb + i;
        w[i] = e < ee ? exp(((double)logits[e0 + e] - M) * inv_t) : 0.0;
        sseg += w[i];
    }
    const double eincl = base1 + wave_scan_incl(sseg, lane);
    const unsigned long long ehit = __ballot(eb < ee && eincl > target);
    if (!ehit) return e0 + len - 1;
    const int el = __ffsll((long long)ehit) - 1;
    int tok = e0 + ee - 1;
    double cum = eincl - sseg;
    bool f = false;
    for (int i = 0; i < 8; ++i) {
        const int e = eb + i;
        if (e < ee && !f) {
            cum += w[i];
            if (cum > target) { tok = e0 + e; f = true; }
        }
    }
    return __shfl(tok, el, WAVE);
}

// Level-2 partials: one wave merges 64 consecutive level-1 partials of one row.
__global__ __launch_bounds__(64) void merge_partials_k(const float *pm, const double *ps, const int32_t *pa, int n1,
                                                       float inv_t, float *pm2, double *ps2, int32_t *pa2, int n2,
                                                       int y_mul, int y_add, const int32_t *y_rows,
                                                       const int32_t *active) {
    if (active != nullptr && *active == 0) return;
    const int j = blockIdx.x, lane = threadIdx.x;
    const size_t row = (size_t)(y_rows != nullptr ? y_rows[blockIdx.y] : (int)blockIdx.y) * y_mul + y_add;
    const int t0 = j * 64, n = min(64, n1 - t0);
    const RowStats r = wave_reduce_partials(pm + row * n1 + t0, ps + row * n1 + t0, pa + row * n1 + t0, n, (double)inv_t, lane);
    if (lane == 0) {
        pm2[row * n2 + j] = (float)r.M;
        ps2[row * n2 + j] = r.S;
        pa2[row * n2 + j] = r.arg;
    }
}

hipError_t launch_merge_partials(const float *pm, const double *ps, const int32_t *pa, int n1, float inv_t, float *pm2,
                                 double *ps2, int32_t *pa2, int rows, int y_mul, int y_add, const int32_t *y_rows,
                                 const int32_t *active, hipStream_t s) {
    const int n2 = (n1 + 63) / 64;
    hipLaunchKernelGGL(merge_partials_k, dim3(n2, rows), dim3(64), 0, s, pm, ps, pa, n1, inv_t, pm2, ps2, pa2, n2, y_mul,
                       y_add, y_rows, active);
    return hipGetLastError();
}

// ---- draft sampling ------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void draft_sample_k(const DraftSampleArgs a) {
    const int b = blockIdx.x, lane = threadIdx.x;
    if (a.st.k[b] == 0) {  // else this sequence stopped drafting earlier in the step
        const int row = b * a.gamma_max + (a.j - 1);
        const PartRow pr = part_row(a.pm, a.ps, a.pa, a.n_tiles, a.tile, a.pm2, a.ps2, a.pa2, a.n2, (size_t)row);
        const float *logits = a.logits + (size_t)row * a.vocab;
        const double inv_t = (double)a.cfg.inv_t;
        const RowStats rs = wave_row_stats(pr, inv_t, lane);
        const int len = a.st.len[b];
        const uint32_t step = (uint32_t)a.st.ctl[0];
        int x;
        if (a.cfg.temperature == 0.f) {
            x = rs.arg;
        } else {
            const double u = philox_uniform(a.cfg.seed, step, (uint32_t)a.j, PURPOSE_DRAFT, (uint32_t)b);
            x = wave_sample_row(logits, a.vocab, pr, rs.M, inv_t, u * rs.S, lane);
        }
        x = min(max(x, 0), a.vocab - 1);  // a row of non-finite logits has no argmax: stay inside the vocabulary
        if (lane == 0) {
            const int pos = len + a.j - 1;
            if (pos < a.st.max_seq) a.st.tokens[(size_t)b * a.st.max_seq + pos] = x;
            a.q_logit[row] = logits[x];
            a.q_max[row] = (float)rs.M;
            a.q_sum[row] = rs.S;
            double conf;
            if (a.cfg.forced) {
                const uint32_t g = (uint32_t)(len - a.st.prompt_len[b] + a.j - 1);
                const double al = (double)a.cfg.alpha[min((int)g, a.cfg.n_alpha - 1)];
                conf = al + (0.5 - philox_uniform(a.cfg.seed, g, 0u, PURPOSE_FORCED, (uint32_t)b)) * 0.5;
                conf = fmin(1.0, fmax(0.0, conf));
            } else {
                conf = 1.0 / rs.S;  // top probability of softmax(l / T_eff)
            }
            const bool stop = (a.cfg.tau > 0.f && conf < (double)a.cfg.tau) || a.j >= a.st.gamma_b[b];
            if (stop) {
                a.st.k[b] = a.j;
                atomicSub(&a.st.ctl[1], 1);
            }
        }
    }
    // the workgroup that arrives last tells the host how many sequences still draft, so that the host launches
    // the next draft pass only when one is needed (a pass whose kernels all return at once still costs its launches)
    if (a.host_pass != nullptr && lane == 0) {
        __threadfence();
        if (atomicAdd(&a.st.ctl[2], 1) == a.st.batch - 1) {
            a.st.ctl[2] = 0;
            const int active = atomicAdd(&a.st.ctl[1], 0);
            const int n = a.st.ctl[3] + 1;
            a.st.ctl[3] = n;
            volatile int32_t *hp = a.host_pass;
            hp[1] = active;
            __threadfence_system();
            hp[0] = n;
        }
    }
}

hipError_t launch_draft_sample(const DraftSampleArgs &a, hipStream_t s) {
    if (a.tile > 512) return hipErrorInvalidValue;
    hipLaunchKernelGGL(draft_sample_k, dim3(a.st.batch), dim3(64), 0, s, a);
    return hipGetLastError();
}

// ---- accept phase ---------------------------------------------------------------------------------
constexpr int ACC_THREADS = 1024;
constexpr int ACC_ROWS_MAX = 65;

__device__ __forceinline__ void commit_step(const AcceptArgs &a, int b, int A, int y) {
    y = min(max(y, 0), a.vocab - 1);
    const int len = a.st.len[b];
    const int pos = len + A;
    if (pos < a.st.max_seq) a.st.tokens[(size_t)b * a.st.max_seq + pos] = y;
    a.st.len[b] = len + A + 1;
    a.y_dev[b] = y;
    a.out_A[b] = A;
    a.out_y[b] = y;
    a.out_k[b] = a.st.k[b];
}

// First row of sequence b in the target's logits and row statistics.
__device__ __forceinline__ size_t target_row0(const AcceptArgs &a, int b, int rows) {
    return a.row_off != nullptr ? (size_t)a.row_off[b] : (size_t)b * rows;
}

__global__ __launch_bounds__(ACC_THREADS) void accept_scan_k(const AcceptArgs a) {
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = a.st.k[b];
    const int rows = a.gamma + 1;
    const double inv_t = (double)a.cfg.inv_t;
    __shared__ double sM[ACC_ROWS_MAX], sS[ACC_ROWS_MAX];
    __shared__ int sArg[ACC_ROWS_MAX];
    __shared__ int sBonus;

    for (int i = wave; i <= k; i += ACC_THREADS / 64) {  // target rows 1..k+1 (0-based i)
        const size_t row = target_row0(a, b, rows) + i;
        const RowStats rs = wave_row_stats(part_row(a.pm, a.ps, a.pa, a.n_tiles, a.tile, a.pm2, a.ps2, a.pa2, a.n2, row),
                                           inv_t, lane);
        if (lane == 0) {
            sM[i] = rs.M; sS[i] = rs.S; sArg[i] = rs.arg;
            a.row_max[row] = rs.M; a.row_sum[row] = rs.S; a.row_arg[row] = rs.arg;
        }
    }
    __syncthreads();
    const int len = a.st.len[b];
    const uint32_t step = (uint32_t)a.st.ctl[0];
    const bool greedy = a.cfg.temperature == 0.f;
    if (wave == 0) {
        // every drafted row is tested by its own lane; A = number of leading passes
        const int g0 = len - a.st.prompt_len[b];
        const int i = lane + 1;
        bool ok = true;
        if (i <= k) {
            const int x = a.st.tokens[(size_t)b * a.st.max_seq + len + i - 1];
            if (a.cfg.forced) {
                const int g = g0 + i - 1;
                const double u = philox_uniform(a.cfg.seed, (uint32_t)g, 0u, PURPOSE_FORCED, (uint32_t)b);
                ok = u < (double)a.cfg.alpha[min(g, a.cfg.n_alpha - 1)];
            } else if (greedy) {
                ok = x == sArg[i - 1];
            } else {
                const size_t prow = target_row0(a, b, rows) + (i - 1);
                const size_t qrow = (size_t)b * a.gamma_max + (i - 1);
                const double p = exp(((double)a.p_logits[prow * a.vocab + x] - sM[i - 1]) * inv_t) / sS[i - 1];
                const double q = exp(((double)a.q_logit[qrow] - (double)a.q_max[qrow]) * inv_t) / a.q_sum[qrow];
                const double u = philox_uniform(a.cfg.seed, step, (uint32_t)i, PURPOSE_ACCEPT, (uint32_t)b);
                ok = u * q < p;
            }
        }
        const unsigned long long fail = __ballot(!ok);
        const int A = fail ? __ffsll((long long)fail) - 1 : k;
        if (lane == 0) {
            a.A_dev[b] = A;
            int resid = 0, bonus = 0;
            if (greedy) {
                a.y_dev[b] = sArg[A];  // row A+1: the refused row, or the bonus row when A == k
            } else if (A == k) {
                bonus = 1;
            } else {
                resid = A + 1;
            }
            a.resid_row[b] = resid;
            sBonus = bonus;
        }
    }
    __syncthreads();
    if (sBonus && wave == 0) {
        const int i = k;  // 0-based bonus row
        const size_t row = target_row0(a, b, rows) + i;
        const double u = philox_uniform(a.cfg.seed, step, (uint32_t)(k + 1), PURPOSE_BONUS, (uint32_t)b);
        const int y = wave_sample_row(a.p_logits + row * a.vocab, a.vocab,
                                      part_row(a.pm, a.ps, a.pa, a.n_tiles, a.tile, a.pm2, a.ps2, a.pa2, a.n2, row), sM[i],
                                      inv_t, u * sS[i], lane);
        if (lane == 0) a.y_dev[b] = y;
    }
}

constexpr int RES_THREADS = 256;
constexpr int RES_EPT_MAX = 16;

// residual weight of vocabulary entry j of the refused row
__device__ __forceinline__ double resid_w(const float *lp, const float *lq, int j, double Mp, double Sp, double Mq,
                                          double Sq, double inv_t) {
    const double p = exp(((double)lp[j] - Mp) * inv_t) / Sp;
    const double q = exp(((double)lq[j] - Mq) * inv_t) / Sq;
    const double d = p - q;
    return d > 0.0 ? d : 0.0;
}

__global__ __launch_bounds__(RES_THREADS) void residual_k(const AcceptArgs a) {
    const int c = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row1 = a.resid_row[b];  // 1-based refused row, 0 when no residual draw is needed
    if (row1 == 0) {
        if (c == 0 && tid == 0) commit_step(a, b, a.A_dev[b], a.y_dev[b]);
        return;
    }
    const int rows = a.gamma + 1;
    const size_t prow = target_row0(a, b, rows) + (row1 - 1);
    const size_t qrow = (size_t)b * a.gamma_max + (row1 - 1);
    const float *lp = a.p_logits + prow * a.vocab;
    const float *lq = a.q_logits + qrow * a.vocab;
    const double Mp = a.row_max[prow], Sp = a.row_sum[prow];
    const double Mq = (double)a.q_max[qrow], Sq = a.q_sum[qrow];
    const double inv_t = (double)a.cfg.inv_t;
    const int NCH = a.n_resid_chunks;
    const int CH = (a.vocab + NCH - 1) / NCH;
    const int EPT = (CH + RES_THREADS - 1) / RES_THREADS;  // <= RES_EPT_MAX (checked on the host)

    __shared__ double wsum[RES_THREADS / 64];
    __shared__ double s_tot;
    __shared__ int s_last;

    // this chunk: contiguous elements per thread, in index order
    auto thread_sum = [&](int chunk, double *keep) {
        const int base = chunk * CH + tid * EPT;
        const int cend = min((chunk + 1) * CH, a.vocab);
        double s = 0.0;
        for (int i = 0; i < EPT; ++i) {
            const int j = base + i;
            const double w = (j < cend) ? resid_w(lp, lq, j, Mp, Sp, Mq, Sq, inv_t) : 0.0;
            if (keep) keep[i] = w;
            s += w;
        }
        return s;
    };
    {
        const double s = thread_sum(c, nullptr);
        const double ws = wave_sum(s);
        if (lane == 0) wsum[wave] = ws;
        __syncthreads();
        if (tid == 0) {
            a.resid_part[(size_t)b * NCH + c] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
            __threadfence();
            const uint32_t t = atomicAdd(&a.ticket[b], 1u);
            s_last = (t == (uint32_t)(NCH - 1));
        }
        __syncthreads();
    }
    if (!s_last) return;
    __threadfence();

    // last workgroup of this sequence: locate the crossing chunk, then the element
    const uint32_t step = (uint32_t)a.st.ctl[0];
    const double u = philox_uniform(a.cfg.seed, step, (uint32_t)row1, PURPOSE_RESID, (uint32_t)b);
    __shared__ int s_chunk, s_y;
    __shared__ double s_base, s_target;
    if (wave == 0) {
        const volatile double *part = a.resid_part + (size_t)b * NCH;
        const int cpl = (NCH + 63) / 64;
        const int cb = lane * cpl, ce = min(cb + cpl, NCH);
        double seg = 0.0;
        for (int i = cb; i < ce; ++i) seg += part[i];
        const double incl = wave_scan_incl(seg, lane);
        const double W = __shfl(incl, 63, WAVE);
        const double target = u * W;
        const unsigned long long hit = __ballot(incl > target && cb < ce);
        int chunk = NCH - 1;
        double base = 0.0;
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;
            double cum = incl - seg;
            int cs = ce - 1;
            double cbse = cum;
            bool f = false;
            for (int i = cb; i < ce; ++i) {
                const double v = part[i];
                if (!f && cum + v > target) { cs = i; cbse = cum; f = true; }
                cum += v;
            }
            if (!f) cbse = cum - part[max(ce - 1, cb)];
            chunk = __shfl(cs, src, WAVE);
            base = __shfl(cbse, src, WAVE);
        }
        if (lane == 0) {
            s_chunk = chunk; s_base = base; s_target = target; s_tot = W;
            s_y = -1;
        }
    }
    __syncthreads();
    if (!(s_tot > 0.0)) {
        // no residual mass (p == q up to rounding): draw from p with the same uniform
        if (wave == 0) {
            const int y = wave_sample_row(lp, a.vocab,
                                          part_row(a.pm, a.ps, a.pa, a.n_tiles, a.tile, a.pm2, a.ps2, a.pa2, a.n2, prow),
                                          Mp, inv_t, u * Sp, lane);
            if (lane == 0) {
                a.ticket[b] = 0;
                commit_step(a, b, a.A_dev[b], y);
            }
        }
        return;
    }
    const int chunk = s_chunk;
    double keep[RES_EPT_MAX];
    const double s = thread_sum(chunk, keep);
    const double incl_w = wave_scan_incl(s, lane);
    if (lane == 63) wsum[wave] = incl_w;
    __syncthreads();
    double off = s_base;
    for (int w = 0; w < wave; ++w) off += wsum[w];
    const double incl = off + incl_w;
    const double target = s_target;
    // first thread whose inclusive sum crosses the target
    __shared__ int s_first;
    if (tid == 0) s_first = RES_THREADS;
    __syncthreads();
    if (incl > target) atomicMin(&s_first, tid);
    __syncthreads();
    const int cend = min((chunk + 1) * CH, a.vocab);
    if (s_first == RES_THREADS) {
        if (tid == 0) s_y = cend - 1;  // rounding left no crossing: last entry of the chunk
    } else if (tid == s_first) {
        double cum = incl - s;
        int y = min(chunk * CH + tid * EPT + EPT, cend) - 1;
        bool f = false;
        for (int i = 0; i < EPT; ++i) {
            const int j = chunk * CH + tid * EPT + i;
            if (j < cend && !f) {
                cum += keep[i];
                if (cum > target) { y = j; f = true; }
            }
        }
        s_y = y;
    }
    __syncthreads();
    if (tid == 0) {
        a.ticket[b] = 0;
        commit_step(a, b, a.A_dev[b], s_y);
    }
}

hipError_t launch_accept(const AcceptArgs &a, hipStream_t s) {
    if (a.gamma + 1 > ACC_ROWS_MAX || a.tile > 512) return hipErrorInvalidValue;
    const int CH = (a.vocab + a.n_resid_chunks - 1) / a.n_resid_chunks;
    if ((CH + RES_THREADS - 1) / RES_THREADS > RES_EPT_MAX) return hipErrorInvalidValue;
    hipLaunchKernelGGL(accept_scan_k, dim3(a.st.batch), dim3(ACC_THREADS), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(residual_k, dim3(a.n_resid_chunks, a.st.batch), dim3(RES_THREADS), 0, s, a);
    return hipGetLastError();
}

// ---- tile partials of caller-provided logits (stand-alone accept, tests) ---------------------------
__global__ __launch_bounds__(64) void row_partials_k(const float *logits, int vocab, int tile, float inv_t, float *pm,
                                                     double *ps, int32_t *pa, int n_tiles) {
    const int t = blockIdx.x, row = blockIdx.y, lane = threadIdx.x;
    const float *l = logits + (size_t)row * vocab;
    const int e0 = t * tile, e1 = min(e0 + tile, vocab);
    float m = -INFINITY;
    int arg = 0x7fffffff;
    for (int e = e0 + lane; e < e1; e += 64) {
        const float v = l[e];
        if (v > m || (v == m && e < arg)) { m = v; arg = e; }
    }
#pragma unroll
    for (int msk = 32; msk >= 1; msk >>= 1) {
        const float om = __shfl_xor(m, msk, WAVE);
        const int oa = __shfl_xor(arg, msk, WAVE);
        if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
    }
    double s = 0.0;
    for (int e = e0 + lane; e < e1; e += 64) s += exp((double)(l[e] - m) * (double)inv_t);
    s = wave_sum(s);
    if (lane == 0) {
        const size_t pi = (size_t)row * n_tiles + t;
        pm[pi] = m; ps[pi] = s; pa[pi] = arg;
    }
}

hipError_t launch_row_partials(const float *logits, int rows, int vocab, int tile, float inv_t, float *pm, double *ps,
                               int32_t *pa, hipStream_t s) {
    const int n_tiles = (vocab + tile - 1) / tile;
    hipLaunchKernelGGL(row_partials_k, dim3(n_tiles, rows), dim3(64), 0, s, logits, vocab, tile, inv_t, pm, ps, pa,
                       n_tiles);
    return hipGetLastError();
}

}  // namespace sd

namespace sd {

// Per drafted row: logit of the drafted token, row max and row sum (what draft_sample_k leaves behind),
// rebuilt from tile partials for callers that bring their own draft logits.
__global__ __launch_bounds__(64) void gather_qstats_k(const float *q_logits, const int32_t *drafted, int vocab,
                                                      const float *pm, const double *ps, const int32_t *pa, int n_tiles,
                                                      float inv_t, float *q_logit, float *q_max, double *q_sum) {
    const int row = blockIdx.x, lane = threadIdx.x;
    const RowStats rs = wave_reduce_partials(pm + (size_t)row * n_tiles, ps + (size_t)row * n_tiles,
                                             pa + (size_t)row * n_tiles, n_tiles, (double)inv_t, lane);
    if (lane == 0) {
        q_logit[row] = q_logits[(size_t)row * vocab + drafted[row]];
        q_max[row] = (float)rs.M;
        q_sum[row] = rs.S;
    }
}

hipError_t launch_gather_qstats(const float *q_logits, const int32_t *drafted, int rows, int vocab, const float *pm,
                                const double *ps, const int32_t *pa, int n_tiles, float inv_t, float *q_logit,
                                float *q_max, double *q_sum, hipStream_t s) {
    hipLaunchKernelGGL(gather_qstats_k, dim3(rows), dim3(64), 0, s, q_logits, drafted, vocab, pm, ps, pa, n_tiles, inv_t,
                       q_logit, q_max, q_sum);
    return hipGetLastError();
}

}  // namespace sd
