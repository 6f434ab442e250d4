// Prompt ingestion and verification of many sequences at once: the same fused projections as the decode
// kernels, for tens to a thousand rows of x, where the work is a dense contraction on the matrix cores rather
// than a weight stream.
//
// One workgroup of four waves (2 x 2) computes a block of 32 WM rows of x by 32 WN rows of W.  Per k-tile
// (32 columns) a stage in LDS holds the operands of the whole block in the register layout of
// v_mfma_f32_16x16x32_bf16:
//   * W tiles come from the re-tiled weights, where a 16-row x 32-column tile is one contiguous KiB that
//     already has that layout;
//   * x is read as fp32 rows, split in registers into two bf16 terms (x = hi + lo, the same split as the
//     decode kernels make) and written as hi and lo fragments.
// Both pass through registers on their way to LDS: the compiler then counts every load exactly and waits for
// the oldest ones only.  (A direct global-to-LDS copy of the W tiles saves the registers, but the compiler
// drains every outstanding load before any LDS access that might alias such a copy, and with it the
// prefetch; measured, that cost more than half of the kernel's time.)  Loads run two iterations ahead of the
// matrix instructions (two sets of staging registers), two workgroups share a compute unit, and the
// block index is mapped so that the workgroups an XCD runs at the same time share their W block (one L2 per
// XCD).  The epilogues are the decode kernels' own arithmetic (RoPE + KV write, residual + next-norm
// statistics, SwiGLU, logits + softmax partials): each wave passes its 32 WM x 32 result tiles through LDS, two
// 16-row groups of W at a time.  A projection with too few blocks to fill the chip shares K out over several
// workgroups per block; gemm_finish_k sums their partial results and applies the epilogue.  8-bit weights
// (q8.hpp) enter as half tiles that are turned into bf16 on the way into LDS.
#include <hip/hip_ext.h>

#include <algorithm>

#include "common.hpp"
#include "epilogue.hpp"
#include "kv.hpp"
#include "params.hpp"
#include "q8.hpp"

namespace sd {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

namespace {

// x = hi + lo with both terms rounded to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ void split4(const f32x4_t v, u32x2_t &hi, u32x2_t &lo) {
    const f32x2_t a = {v[0], v[1]}, b = {v[2], v[3]};
    const bf16x2_t ha = __builtin_convertvector(a, bf16x2_t), hb = __builtin_convertvector(b, bf16x2_t);
    const bf16x2_t la = __builtin_convertvector(a - __builtin_convertvector(ha, f32x2_t), bf16x2_t);
    const bf16x2_t lb = __builtin_convertvector(b - __builtin_convertvector(hb, f32x2_t), bf16x2_t);
    hi.x = __builtin_bit_cast(uint32_t, ha);
    hi.y = __builtin_bit_cast(uint32_t, hb);
    lo.x = __builtin_bit_cast(uint32_t, la);
    lo.y = __builtin_bit_cast(uint32_t, lb);
}

}  // namespace

constexpr int GEMM_TS = 36;                      // row stride (floats) of a wave's result tile in the epilogue

// Loads run two iterations ahead in both forms (two sets of staging registers).  DEEP: the fragments of the next
// iteration are read while this one multiplies (double-buffered in registers as well); otherwise they are read where
// they are used, which fits the registers of the wide block.
template <int WM, int WN, bool DEEP, int MW>
struct GemmShape {
    static constexpr int NWAVES = 2 * MW;           // MW x 2 waves, each 16 WM rows of x by 16 WN rows of W
    static constexpr int THREADS = 64 * NWAVES;
    static constexpr int BMB = MW * WM;             // 16-row blocks of x per workgroup
    static constexpr int BNG = 2 * WN;              // 16-row groups of W per workgroup
    static constexpr int XS = BMB * 2 * 1024;       // bytes of the x fragments of a stage (hi and lo)
    static constexpr int WS = BNG * 1024;           // bytes of the W tiles of a stage
    static constexpr int XI = 2 * BMB / NWAVES;     // x loads per thread and stage
    static constexpr int WI = BNG / NWAVES;         // W loads per thread and stage
    static constexpr int RING = 2 * (XS + WS);      // two stages alternate
    static constexpr int EPI_BYTES = NWAVES * (WM * 16 * GEMM_TS + WM * 16) * 4;  // per wave: result tile + row scales
    static constexpr int LDS = RING > EPI_BYTES ? RING : EPI_BYTES;
};

// The workgroup meets once this wave's LDS traffic is done.  (__syncthreads would also drain every global
// load and with it the prefetch.)
__device__ __forceinline__ void stage_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int WM, int WN> struct GemmFrags { u32x4_t ah[WM], al[WM], bw[WN]; };

// k-tiles per share when K is shared out over `shares` workgroups (8-bit weights: whole 64-k tiles, i.e. even)
__host__ __device__ inline int share_ktiles(int KT, int shares, int q8) {
    const int n = (KT + shares - 1) / shares;
    return q8 ? n + (n & 1) : n;
}

// The arguments of a projection as seen from row `row0`: the epilogues index rows from zero.
template <int EPI> __device__ __forceinline__ GemvArgs rows_from(const GemvArgs &a, int row0) {
    GemvArgs b = a;
    const size_t ro = (size_t)row0;
    if constexpr (EPI == EPI_PLAIN) {
        b.y += ro * a.n0;
    } else if constexpr (EPI == EPI_RESID) {
        b.xres += ro * a.n0; b.xg += ro * a.n0; b.xgb += ro * a.n0; b.ssq_out += ro * a.ssq_stride;
    } else if constexpr (EPI == EPI_SWIGLU) {
        b.y += ro * a.n0; b.yb += ro * a.n0;
    } else if constexpr (EPI == EPI_QKV) {
        b.y += ro * a.nq * a.hd; b.yb += ro * a.nq * a.hd; b.row_pos += row0; b.row_seq += row0;
    } else if constexpr (EPI == EPI_LOGITS) {
        if (a.y_rows != nullptr) {
            b.y_rows += row0;  // the rows' own output rows, looked up by the epilogue
        } else {
            const size_t orow = ro * a.y_mul;
            b.y += orow * a.y_stride; b.pm += orow * a.n_tiles; b.ps += orow * a.n_tiles; b.pa += orow * a.n_tiles;
        }
    }
    return b;
}

// QKV epilogue of one wave over ROWS rows x two groups (16 RoPE pairs) of its result tile, with every load that
// does not depend on the tile issued first: the caller fetched each row's position and KV page once per wave
// (rows_pos / rows_page, row step `it` = rows 4 it + lane / 16), the rotary factors of this lane's pair are fetched
// here for all its rows before the first of them is used.  Same arithmetic as epilogue_tile<EPI_QKV>.
template <int ROWS>
__device__ __forceinline__ void qkv_wave_epilogue(const GemvArgs &b, const float *tile, int TS, const float *scale, int Rw,
                                                  int g, int n_groups, int Ntot, int lane, const int (&rows_pos)[ROWS / 4],
                                                  const int (&rows_page)[ROWS / 4]) {
    constexpr int NI = ROWS / 4;
    const int rsub = lane >> 4, p = lane & 15, h = p >> 3, pj = p & 7;
    if (g + h >= n_groups) return;  // the second group of the pass lies beyond the matrix: no shuffles below
    const int half = b.hd >> 1;
    const int P = (g + h) * 8 + pj;
    if (P >= (Ntot >> 1)) return;
    const int hh = P / half, j = P % half;
    const bool rot = hh < b.nq + b.nkv;
    float cs[NI], sn[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        cs[it] = 1.f; sn[it] = 0.f;
        if (rot && it * 4 + rsub < Rw) {
            cs[it] = b.rope_cos[(size_t)rows_pos[it] * half + j];
            sn[it] = b.rope_sin[(size_t)rows_pos[it] * half + j];
        }
    }
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int r = it * 4 + rsub;
        if (r >= Rw) continue;
        const float a1 = tile[r * TS + h * 16 + pj] * scale[r];
        const float a2 = tile[r * TS + h * 16 + 8 + pj] * scale[r];
        const float y1 = rot ? a1 * cs[it] - a2 * sn[it] : a1;
        const float y2 = rot ? a2 * cs[it] + a1 * sn[it] : a2;
        if (hh < b.nq) {
            const size_t o = (size_t)r * b.nq * b.hd + (size_t)hh * b.hd + j;
            b.y[o] = y1;
            b.y[o + half] = y2;
            store_split_bf16(b.yb, o, b.yb_lo, y1);
            store_split_bf16(b.yb, o + half, b.yb_lo, y2);
        } else {
            const bool is_k = hh < b.nq + b.nkv;
            const int kvh = hh - b.nq - (is_k ? 0 : b.nkv);
            const int in_page = rows_pos[it] & (b.kv.page_tokens - 1);
            const size_t base = kv_head_base(b.kv, rows_page[it], kvh);
            const size_t e1 = base + (is_k ? kv_in_k(b.kv, in_page, j) : kv_in_v(b.kv, in_page, j));
            const size_t e2 = base + (is_k ? kv_in_k(b.kv, in_page, j + half) : kv_in_v(b.kv, in_page, j + half));
            void *pool = is_k ? b.kv.k : b.kv.v;
            if (b.kv_dtype == DT_BF16) {
                reinterpret_cast<bf16_t *>(pool)[e1] = f32_to_bf16(y1);
                reinterpret_cast<bf16_t *>(pool)[e2] = f32_to_bf16(y2);
            } else {
                reinterpret_cast<float *>(pool)[e1] = y1;
                reinterpret_cast<float *>(pool)[e2] = y2;
            }
        }
    }
}

// positions and KV pages of a wave's rows for qkv_wave_epilogue (b: arguments seen from the wave's first row)
template <int ROWS>
__device__ __forceinline__ void qkv_wave_rows(const GemvArgs &b, int Rw, int lane, int (&rows_pos)[ROWS / 4],
                                              int (&rows_page)[ROWS / 4]) {
#pragma unroll
    for (int it = 0; it < ROWS / 4; ++it) {
        const int r = it * 4 + (lane >> 4);
        rows_pos[it] = 0;
        rows_page[it] = 0;
        if (r < Rw) {
            rows_pos[it] = b.row_pos[r];
            rows_page[it] = kv_page(b.kv, b.row_seq[r], rows_pos[it]);
        }
    }
}

// scale[r] = rsqrt(mean(x_r^2) + eps) from the statistics slots of the producer: one wave per row.
__global__ __launch_bounds__(256) void row_scale_k(const float *ssq, int slots, int stride, int R, int K, float eps,
                                                   float *scale) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (r >= R) return;
    float s = 0.f;
    for (int q = lane; q < slots; q += 64) s += ssq[(size_t)r * stride + q];
    s = wave_sum(s);
    if (lane == 0) scale[r] = rsqrtf(s / (float)K + eps);
}

// Arguments as for the decode kernels, except: x is a.x (fp32, row-major, row length K, x_mul = 1, x_add = 0) and the
// row scales come ready-made in a.row_scale (null: ones).  grid.x = 8 * ceil(n_blocks / 8) * m_blocks * ksplit.
//
// Timeline of the deep main loop (iteration t multiplies k-tile t from fragments already in registers):
//   barrier            stage t + 1 is complete in LDS; nobody reads stage t any more
//   stash   t + 2      from the registers loaded two iterations ago into the slot stage t has left (x is split here)
//   issue   t + 4      global loads into the registers just freed
//   read    t + 1      fragments for the next iteration
//   multiply t
// Stages past the last k-tile repeat it into slots nobody reads again, which keeps the loop uniform.
// WQ: 1 = 8-bit weights (q8.hpp).  A k-tile of the loop is then half of a 64-k weight tile: the lane's first or
// second eight bytes, turned into bf16 on the way into LDS, and the x fragments gather the matching k sets (chunk c
// of k-tile t holds k = 64 (t / 2) + 16 c + 8 (t % 2) .. + 8).  The column scales multiply the result tile.
// MW: wave rows of the workgroup (2: four waves, blocks of 32 WM rows of x; 4: eight waves, 64 WM rows, one
// workgroup per compute unit - a third fewer bytes fetched per matrix instruction than the wide four-wave block).
template <int EPI, int WM, int WN, bool DEEP, int WQ, int MW>
__global__ __launch_bounds__((GemmShape<WM, WN, DEEP, MW>::THREADS), 2) void gemm_mfma_k(
    const GemvArgs a, const int m_blocks, const int ksplit, const int64_t split_stride) {
    using S = GemmShape<WM, WN, DEEP, MW>;
    constexpr int XI = S::XI;
    if (a.active != nullptr && *a.active == 0) return;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // the wave index is a scalar: every branch around a matrix instruction must be a scalar branch
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    int Ntot = a.n0;
    if (EPI == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (EPI == EPI_SWIGLU) Ntot = 2 * a.n0;
    const int n_groups = Ntot >> 4;
    const int n_blocks = (n_groups + S::BNG - 1) / S::BNG;
    // consecutive workgroup ids go round the XCDs: the m_blocks row blocks of one W block stay on one XCD
    // ksplit > 1 (plain epilogue only): the workgroup multiplies its share of the k-tiles and leaves a partial
    // result in slab ks of a.y (slabs split_stride floats apart) for gemm_finish_k
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int ks = j % ksplit, jm = j / ksplit;
    const int nb = (jm / m_blocks) * 8 + xcd, mb = jm % m_blocks;
    if (nb >= n_blocks) return;
    const int g0 = nb * S::BNG, m0 = mb * S::BMB * 16;
    const int K = a.K, R = a.R;
    const int KTall = K >> 5, KTs = share_ktiles(KTall, ksplit, WQ);
    const int kt0 = ks * KTs, KT = min(KTall, kt0 + KTs) - kt0;  // the host leaves no share empty
    char *const xs = smem;               // [2][XS]
    char *const ws = smem + 2 * S::XS;   // [2][WS]

    // ---- load plan -------------------------------------------------------------------------------------
    // W: wave w moves the tiles w, w + NWAVES, ... of the stage
    const char *wsrc[S::WI];
#pragma unroll
    for (int i = 0; i < S::WI; ++i) {
        const int g = min(g0 + wave + S::NWAVES * i, n_groups - 1);
        // 16-bit: tile (g, kt) of 1 KiB; 8-bit: k-tile kt is half kt % 2 of tile (g, kt / 2) (the host keeps kt0 even)
        wsrc[i] = reinterpret_cast<const char *>(a.w0) + (WQ ? ((size_t)g * (KTall >> 1) + (kt0 >> 1)) * 1024 : ((size_t)g * KTall + kt0) * 1024) +
                  lane * 16;
    }
    // x: the block's fragments are filled in units of 512 contiguous bytes (16 rows x two k-chunks of 8 columns), one
    // unit per wave-wide load, so that the LDS writes of a wave touch every bank once: unit q = XI wave + i is row
    // block q / 2, k-chunks 2 (q % 2) and 2 (q % 2) + 1; lane l holds row l / 2 % 16, k-chunk l / 32 of the pair,
    // elements 4 (l % 2) ..+4, and its eight bytes (per term) land at 8 l of the unit.  Two consecutive loads of a
    // wave read the two halves of the same 128-byte lines.
    const float *xsrc[XI];
    int xdst[XI];
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        const int q = XI * wave + i, rb = q >> 1, c = 2 * (q & 1) + (lane >> 5);
        const int row = m0 + rb * 16 + ((lane >> 1) & 15);
        xsrc[i] = a.x + (size_t)min(row, R - 1) * K + (size_t)kt0 * 32 + (8 << WQ) * c + 4 * (lane & 1);
        xdst[i] = rb * 2048 + (q & 1) * 512 + lane * 8;
    }

    f32x4_t acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int n = 0; n < WN; ++n) acc[i][n] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    struct Staged { f32x4_t x[XI]; u32x4_t w[S::WI]; };  // 8-bit weights use half of each w
    auto issue = [&](int stage, Staged &r) {
        const int kt = min(stage, KT - 1);
#pragma unroll
        for (int i = 0; i < S::WI; ++i) {
            if constexpr (WQ) {
                const q8_u32x2_t h = *reinterpret_cast<const q8_u32x2_t *>(wsrc[i] + (size_t)(kt >> 1) * 1024 + (kt & 1) * 8);
                r.w[i] = u32x4_t{h.x, h.y, 0u, 0u};
            } else {
                r.w[i] = *reinterpret_cast<const u32x4_t *>(wsrc[i] + (size_t)kt * 1024);
            }
        }
        // 8-bit weights: k-tile kt starts at 64 (kt / 2) + 8 (kt % 2) and its chunks are 16 columns apart
        const size_t xo = WQ ? (size_t)(kt >> 1) * 64 + (kt & 1) * 8 : (size_t)kt * 32;
#pragma unroll
        for (int i = 0; i < XI; ++i) r.x[i] = *reinterpret_cast<const f32x4_t *>(xsrc[i] + xo);
    };
    auto stash = [&](const Staged &r, int slot) {
        char *xslot = xs + slot * S::XS, *wslot = ws + slot * S::WS;
#pragma unroll
        for (int i = 0; i < XI; ++i) {
            u32x2_t hi, lo;
            split4(r.x[i], hi, lo);
            *reinterpret_cast<u32x2_t *>(xslot + xdst[i]) = hi;
            *reinterpret_cast<u32x2_t *>(xslot + xdst[i] + 1024) = lo;
        }
#pragma unroll
        for (int i = 0; i < S::WI; ++i)
            *reinterpret_cast<u32x4_t *>(wslot + (wave + S::NWAVES * i) * 1024 + lane * 16) =
                WQ ? q8_half_to_bf16(q8_u32x2_t{r.w[i].x, r.w[i].y}) : r.w[i];
    };
    auto read = [&](int stage, GemmFrags<WM, WN> &f) {
        const char *xslot = xs + (stage & 1) * S::XS + lane * 16;
        const char *wslot = ws + (stage & 1) * S::WS + lane * 16;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            f.ah[i] = *reinterpret_cast<const u32x4_t *>(xslot + (wm * WM + i) * 2048);
            f.al[i] = *reinterpret_cast<const u32x4_t *>(xslot + (wm * WM + i) * 2048 + 1024);
        }
#pragma unroll
        for (int n = 0; n < WN; ++n) f.bw[n] = *reinterpret_cast<const u32x4_t *>(wslot + (wn * WN + n) * 1024);
    };
    auto multiply = [&](const GemmFrags<WM, WN> &f) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
#pragma unroll
            for (int n = 0; n < WN; ++n) {
                acc[i][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, f.ah[i]),
                                                                    __builtin_bit_cast(bf16x8_t, f.bw[n]), acc[i][n], 0, 0, 0);
                acc[i][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, f.al[i]),
                                                                    __builtin_bit_cast(bf16x8_t, f.bw[n]), acc[i][n], 0, 0, 0);
            }
        }
    };

    Staged r0, r1;
    GemmFrags<WM, WN> fa, fb;
    if constexpr (DEEP) {
        issue(0, r0);
        issue(1, r1);
        stash(r0, 0);
        issue(2, r0);
        stage_barrier();  // stage 0 complete
        stash(r1, 1);
        issue(3, r1);
        read(0, fa);
        for (int t = 0; t + 1 < KT; t += 2) {  // two iterations per trip: registers and slots alternate
            stage_barrier();
            stash(r0, 0);
            issue(t + 4, r0);
            read(t + 1, fb);
            multiply(fa);
            stage_barrier();
            stash(r1, 1);
            issue(t + 5, r1);
            read(t + 2, fa);
            multiply(fb);
        }
        if (KT & 1) multiply(fa);  // the last k-tile of an odd count was read by the trip before
    } else {
        // iteration t: issue t + 2, read and multiply t, stash t + 1 (loaded an iteration ago), meet
        issue(0, r0);
        issue(1, r1);
        stash(r0, 0);
        stage_barrier();
        for (int t = 0; t + 1 < KT; t += 2) {  // two iterations per trip: the staging registers alternate
            issue(t + 2, r0);
            read(t, fa);
            multiply(fa);
            stash(r1, 1);
            stage_barrier();
            issue(t + 3, r1);
            read(t + 1, fa);
            multiply(fa);
            stash(r0, 0);
            stage_barrier();
        }
        if (KT & 1) {
            read(KT - 1, fa);
            multiply(fa);
        }
    }
    __syncthreads();  // every load has landed and every wave has left the stages before they are reused

    // ---- epilogue: this wave's rows m0 + 16 WM wm ..+16 WM, two groups of W (32 columns) at a time ----------
    constexpr int TS = GEMM_TS;
    float *tile = reinterpret_cast<float *>(smem) + wave * (WM * 16 * TS + WM * 16);
    float *scale = tile + WM * 16 * TS;
    const int row0 = m0 + wm * WM * 16;
    const int Rw = max(0, min(WM * 16, R - row0));
    for (int r = lane; r < WM * 16; r += 64) scale[r] = (a.row_scale != nullptr && r < Rw) ? a.row_scale[row0 + r] : 1.f;
    GemvArgs b = rows_from<EPI>(a, row0);  // the same arguments, seen from this wave's first row
    if constexpr (EPI == EPI_PLAIN) b.y += (size_t)ks * split_stride;
    // the tile and the scales are private to the wave: LDS serves a wave's accesses in order, so a wave-level
    // wait orders its writes before its reads
    auto wave_sync = [] { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); };
    int rows_pos[WM * 4], rows_page[WM * 4];  // QKV: positions and KV pages of this lane's rows
    if constexpr (EPI == EPI_QKV) qkv_wave_rows<WM * 16>(b, Rw, lane, rows_pos, rows_page);
    constexpr int RI = WM;  // residual epilogue: row steps (8 rows each) of half a pass
#pragma unroll
    for (int p = 0; p < WN / 2; ++p) {
        const int g = g0 + wn * WN + 2 * p;  // first group of the pass
        // residual: a lane owns four columns of one row per row step; the residual values of half the rows are
        // fetched before the tile is staged, those of the other half while the first is worked through
        const int rsub = lane >> 3, c4 = (lane & 7) * 4;
        const int gl = g + (c4 >> 4);
        const bool col_ok = gl < n_groups;
        const int n = g * 16 + c4;
        f32x4_t xo[RI], gn = {1.f, 1.f, 1.f, 1.f};
        auto fetch = [&](int half) {
#pragma unroll
            for (int it = 0; it < RI; ++it) {
                const int r = (half * RI + it) * 8 + rsub;
                xo[it] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                if (col_ok && r < Rw) xo[it] = *reinterpret_cast<const f32x4_t *>(b.xres + (size_t)r * a.n0 + n);
            }
        };
        if constexpr (EPI == EPI_RESID) {
            if (col_ok && a.g_next != nullptr) gn = *reinterpret_cast<const f32x4_t *>(a.g_next + n);
            fetch(0);
        }
        // 8-bit weights: the scales of this lane's two columns of the pass (a partial result of a shared-out K is
        // scaled by gemm_finish_k instead)
        float wcs[2] = {1.f, 1.f};
        if (WQ && a.wscale != nullptr) {
#pragma unroll
            for (int h = 0; h < 2; ++h) wcs[h] = a.wscale[(size_t)min(g + h, n_groups - 1) * 16 + (lane & 15)];
        }
        wave_sync();  // the previous pass has read the tile
        // register v of lane l is x row 4 (l / 16) + v, W row l % 16
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    tile[(i * 16 + (lane >> 4) * 4 + v) * TS + h * 16 + (lane & 15)] = WQ ? acc[i][2 * p + h][v] * wcs[h] : acc[i][2 * p + h][v];
        wave_sync();
        if constexpr (EPI == EPI_RESID) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                if (half == 1) fetch(1);
#pragma unroll
                for (int it = 0; it < RI; ++it) {
                    const int r = (half * RI + it) * 8 + rsub;
                    const bool ok = col_ok && r < Rw;
                    const f32x4_t y = *reinterpret_cast<const f32x4_t *>(tile + r * TS + c4);
                    const float sc = scale[r];
                    f32x4_t xn, xg;
                    float sq = 0.f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        xn[e] = xo[it][e] + y[e] * sc;
                        xg[e] = xn[e] * gn[e];
                        sq += xn[e] * xn[e];
                    }
                    if (ok) {
                        const size_t o = (size_t)r * a.n0 + n;
                        *reinterpret_cast<f32x4_t *>(b.xres + o) = xn;
                        *reinterpret_cast<f32x4_t *>(b.xg + o) = xg;
                        u32x2_t hi, lo;
                        split4(xg, hi, lo);
                        *reinterpret_cast<u32x2_t *>(b.xgb + o) = hi;
                        if (a.xgb_lo) *reinterpret_cast<u32x2_t *>(b.xgb + o + a.xgb_lo) = lo;
                    }
                    sq += __shfl_xor(sq, 1, WAVE);
                    sq += __shfl_xor(sq, 2, WAVE);
                    if (ok && (lane & 3) == 0) b.ssq_out[(size_t)r * a.ssq_stride + gl] = sq;
                }
            }
        } else if constexpr (EPI == EPI_QKV) {
            if (g < n_groups && Rw > 0) qkv_wave_epilogue<WM * 16>(b, tile, TS, scale, Rw, g, n_groups, Ntot, lane, rows_pos, rows_page);
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h)
                if (g + h < n_groups && Rw > 0) epilogue_tile<EPI, 16, 64>(b, tile + h * 16, TS, scale, Rw, g + h, Ntot, lane);
        }
    }
}

// Second half of a projection whose k-tiles were shared out: sums the ksplit partial results in slab order (the
// result does not depend on which workgroup finished first) and applies the epilogue.  One workgroup per 16-row
// group of W and 64 rows of x, one wave per 16 rows.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_finish_k(const GemvArgs a, const float *part, const int ksplit,
                                                     const int64_t split_stride) {
    if (a.active != nullptr && *a.active == 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int Ntot = a.n0;
    if (EPI == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (EPI == EPI_SWIGLU) Ntot = 2 * a.n0;
    const int g = blockIdx.x, row0 = blockIdx.y * 64 + wave * 16;
    const int Rw = max(0, min(16, a.R - row0));
    __shared__ __attribute__((aligned(16))) float tiles[4][16 * 20];
    __shared__ float scales[4][16];
    float *tile = tiles[wave], *scale = scales[wave];
    const GemvArgs b = rows_from<EPI>(a, row0);
    int rows_pos[4], rows_page[4];  // QKV: positions and KV pages of this lane's rows, in flight beside the partial sums
    if constexpr (EPI == EPI_QKV) qkv_wave_rows<16>(b, Rw, lane, rows_pos, rows_page);
    const int r = lane >> 2, c4 = (lane & 3) * 4;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    // residual form: a lane's four sums meet its four residual values directly, so everything it needs - residual,
    // next norm's gains, row scale, the slabs - is requested at once and the kernel is one round of loads deep
    f32x4_t xo = {0.f, 0.f, 0.f, 0.f}, gn = {1.f, 1.f, 1.f, 1.f};
    float sc = 1.f;
    if constexpr (EPI == EPI_RESID) {
        if (r < Rw) {
            xo = *reinterpret_cast<const f32x4_t *>(b.xres + (size_t)r * a.n0 + g * 16 + c4);
            if (a.g_next != nullptr) gn = *reinterpret_cast<const f32x4_t *>(a.g_next + g * 16 + c4);
            if (a.row_scale != nullptr) sc = a.row_scale[row0 + r];
        }
    }
    if (r < Rw) {
        const float *p = part + (size_t)(row0 + r) * Ntot + g * 16 + c4;
        // eight slabs in flight at a time (a loop of dependent load-and-add rounds costs a memory latency per slab);
        // slab indices past the last one re-read it and are left out of the sum, which stays in slab order
        for (int s0 = 0; s0 < ksplit; s0 += 8) {
            f32x4_t v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = *reinterpret_cast<const f32x4_t *>(p + (size_t)min(s0 + i, ksplit - 1) * split_stride);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (s0 + i < ksplit) { acc[0] += v[i][0]; acc[1] += v[i][1]; acc[2] += v[i][2]; acc[3] += v[i][3]; }
            }
        }
        if (a.wscale != nullptr) {  // 8-bit weights: the column scales
            const f32x4_t sc = *reinterpret_cast<const f32x4_t *>(a.wscale + (size_t)g * 16 + c4);
            acc[0] *= sc[0]; acc[1] *= sc[1]; acc[2] *= sc[2]; acc[3] *= sc[3];
        }
    }
    if constexpr (EPI == EPI_RESID) {
        const bool ok = r < Rw;
        f32x4_t xn, xg;
        float sq = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            xn[e] = xo[e] + acc[e] * sc;
            xg[e] = xn[e] * gn[e];
            sq += xn[e] * xn[e];
        }
        if (ok) {
            const size_t o = (size_t)r * a.n0 + g * 16 + c4;
            *reinterpret_cast<f32x4_t *>(b.xres + o) = xn;
            *reinterpret_cast<f32x4_t *>(b.xg + o) = xg;
            u32x2_t hi, lo;
            split4(xg, hi, lo);
            *reinterpret_cast<u32x2_t *>(b.xgb + o) = hi;
            if (a.xgb_lo) *reinterpret_cast<u32x2_t *>(b.xgb + o + a.xgb_lo) = lo;
        }
        sq += __shfl_xor(sq, 1, WAVE);
        sq += __shfl_xor(sq, 2, WAVE);
        if (ok && (lane & 3) == 0) b.ssq_out[(size_t)r * a.ssq_stride + g] = sq;
        return;
    }
    *reinterpret_cast<f32x4_t *>(tile + r * 20 + c4) = acc;
    if (lane < 16) scale[lane] = (a.row_scale != nullptr && lane < Rw) ? a.row_scale[row0 + lane] : 1.f;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the tile is private to the wave
    if (Rw > 0) {
        // (the QKV form works on pairs of groups: told that the matrix ends after this one, it leaves the second alone)
        if constexpr (EPI == EPI_QKV) qkv_wave_epilogue<16>(b, tile, 20, scale, Rw, g, g + 1, Ntot, lane, rows_pos, rows_page);
        else epilogue_tile<EPI, 16, 64>(b, tile, 20, scale, Rw, g, Ntot, lane);
    }
}

template <int EPI, int WM, int WN, bool DEEP, int WQ, int MW = 2>
static hipError_t launch_gemm_one(const GemvArgs &a, int Ntot, int ksplit, int64_t split_stride, hipEvent_t ev0, hipEvent_t ev1,
                                  hipStream_t s) {
    using S = GemmShape<WM, WN, DEEP, MW>;
    const int n_blocks = (Ntot / 16 + S::BNG - 1) / S::BNG;
    const int m_blocks = (a.R + S::BMB * 16 - 1) / (S::BMB * 16);
    const int grid = ((n_blocks + 7) / 8) * 8 * m_blocks * ksplit;
    static bool attr_set = false;  // per instantiation
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_mfma_k<EPI, WM, WN, DEEP, WQ, MW>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, S::LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (ev0 != nullptr)
        hipExtLaunchKernelGGL((gemm_mfma_k<EPI, WM, WN, DEEP, WQ, MW>), dim3(grid), dim3(S::THREADS), S::LDS, s, ev0, ev1, 0, a, m_blocks,
                              ksplit, split_stride);
    else
        hipLaunchKernelGGL((gemm_mfma_k<EPI, WM, WN, DEEP, WQ, MW>), dim3(grid), dim3(S::THREADS), S::LDS, s, a, m_blocks, ksplit,
                           split_stride);
    return hipGetLastError();
}

// Shares of K for a projection whose blocks would leave most compute units idle: a workgroup's time is its k-tiles
// times the load latency it cannot hide (about 0.6 us per k-tile), whatever the rows, so a matrix with few blocks
// (N = d_model at up to a few hundred rows) is served faster by more, shorter workgroups plus one summing pass.
static int pick_ksplit(int Ntot, int K, int R, size_t ws_bytes, bool q8) {
    const int wgs = ((Ntot + 127) / 128) * ((R + 127) / 128), KT = K / 32;
    if (wgs > 128 || KT < 8) return 1;
    int sp = std::min(std::min(8, 256 / wgs), KT / 4);
    while (sp > 1 && (size_t)sp * R * Ntot * sizeof(float) > ws_bytes) --sp;
    while (sp > 1 && (sp - 1) * share_ktiles(KT, sp, q8) >= KT) --sp;  // no empty share
    return std::max(sp, 1);
}

template <int EPI>
static hipError_t launch_gemm_cfg(const GemvArgs &a, int Ntot, int forced, float *ws, size_t ws_bytes, hipEvent_t ev0,
                                  hipEvent_t ev1, hipStream_t s) {
    const bool q8 = a.wscale != nullptr;
    if (q8 && a.K % 64) return hipErrorInvalidValue;
    int cfg = forced % 1000, ksplit = forced / 1000;
    const int KT = a.K / 32;
    auto shares_ok = [&](int sp) {
        return sp <= KT && (sp - 1) * share_ktiles(KT, sp, q8) < KT && ws != nullptr &&
               (size_t)sp * a.R * Ntot * sizeof(float) <= ws_bytes;
    };
    if (cfg == 0) {
        // all shapes are bound by what a compute unit can fetch per matrix instruction: the 256 x 256 block of eight
        // waves needs the least (measured 5-8 % ahead of the wide four-wave block once it fills the chip), the
        // narrow block fills the chip when the wider ones would leave compute units idle
        const int m_blocks = (a.R + 127) / 128;
        const int wg8 = ((Ntot + 255) / 256) * ((a.R + 255) / 256);
        // (not when its 256-row blocks would leave the last band of rows half empty: up to 128 rows, 257-384, ... the
        // 128-row blocks do a quarter or more less work; measured on the LM head at 100 rows 267 against 411 us)
        if (wg8 >= 256 && (m_blocks % 2 == 0 || m_blocks >= 7)) {
            cfg = 808;
        } else if (ksplit == 0 && wg8 <= 128 && a.R >= 256 && KT >= 320) {
            // few 256 x 256 blocks, many rows and a long K (the down projection at prefill sizes): the big block with
            // K shared out fetches half of what the narrow block would for the same work (measured 285 -> 233 us at
            // K = 14336; at K <= 8192 the summing pass eats the gain)
            int sp = std::min(std::min(8, 256 / wg8), KT / 4);
            while (sp > 1 && !shares_ok(sp)) --sp;
            if (sp > 1) { cfg = 808; ksplit = sp; }
        }
        if (cfg == 0) cfg = ((Ntot + 255) / 256) * m_blocks > 256 ? 408 : 404;
        // up to 96 rows the narrow block is 96 rows high, up to 64 rows 64, up to 32 rows 32: fewer matrix
        // instructions and fragment reads per k-tile (measured on every projection shape of the 8B and 1B models:
        // 8-15 % faster at 96 rows, 20-30 % at 64, a further 12-18 % at 32)
        if ((cfg == 404 || cfg == 408) && a.R <= 64) cfg = a.R <= 32 ? 104 : 204;
        // (the 96-row block also wherever it needs no more blocks than the 128-row one: 129-192 rows, 257-288)
        if (cfg == 404 && (a.R + 95) / 96 == (a.R + 127) / 128) cfg = 304;
        // 97-128 rows (one 128-row block): eight waves of 32 x 64 on the 128 x 128 block where the matrix gives every
        // compute unit a block (measured, gate/up shape at 128 rows: 87 -> 71 us), else two 64-row blocks, which make
        // twice the workgroups (down / QKV / output projection shapes: 57 -> 51, 35 -> 32, 30 -> 27 us)
        if (cfg == 404 && a.R > 96 && a.R <= 128 && !q8) cfg = (Ntot + 127) / 128 >= 200 ? 524 : 204;
    }
    if (ksplit == 0) ksplit = ((cfg == 404 || cfg == 304 || cfg == 204 || cfg == 104) && ws != nullptr) ? pick_ksplit(Ntot, a.K, a.R, ws_bytes, q8) : 1;
    if (ksplit > 1) {
        if (!shares_ok(ksplit)) return hipErrorInvalidValue;
        const int64_t stride = (int64_t)a.R * Ntot;
        GemvArgs p = a;  // partial results: plain rows of Ntot columns, unscaled
        p.n0 = Ntot; p.y = ws; p.row_scale = nullptr; p.ssq_in = nullptr; p.wscale = nullptr;
        hipError_t e = hipErrorInvalidValue;
        switch (cfg + 1000 * (int)q8) {
            case 404: e = launch_gemm_one<EPI_PLAIN, 4, 4, true, 0>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 204: e = launch_gemm_one<EPI_PLAIN, 2, 4, true, 0>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 304: e = launch_gemm_one<EPI_PLAIN, 3, 4, true, 0>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 1304: e = launch_gemm_one<EPI_PLAIN, 3, 4, true, 1>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 104: e = launch_gemm_one<EPI_PLAIN, 1, 4, true, 0>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 1104: e = launch_gemm_one<EPI_PLAIN, 1, 4, true, 1>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 1204: e = launch_gemm_one<EPI_PLAIN, 2, 4, true, 1>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 1404: e = launch_gemm_one<EPI_PLAIN, 4, 4, true, 1>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 408: e = launch_gemm_one<EPI_PLAIN, 4, 8, false, 0>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 1408: e = launch_gemm_one<EPI_PLAIN, 4, 8, false, 1>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 808: e = launch_gemm_one<EPI_PLAIN, 4, 8, false, 0, 4>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 524: e = launch_gemm_one<EPI_PLAIN, 2, 4, true, 0, 4>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
            case 1808: e = launch_gemm_one<EPI_PLAIN, 4, 8, false, 1, 4>(p, Ntot, ksplit, stride, ev0, ev1, s); break;
        }
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((gemm_finish_k<EPI>), dim3(Ntot / 16, (a.R + 63) / 64), dim3(256), 0, s, a, ws, ksplit, stride);
        return hipGetLastError();
    }
    switch (cfg + 1000 * (int)q8) {
        case 408: return launch_gemm_one<EPI, 4, 8, false, 0>(a, Ntot, 1, 0, ev0, ev1, s);
        case 404: return launch_gemm_one<EPI, 4, 4, true, 0>(a, Ntot, 1, 0, ev0, ev1, s);
        case 204: return launch_gemm_one<EPI, 2, 4, true, 0>(a, Ntot, 1, 0, ev0, ev1, s);
        case 304: return launch_gemm_one<EPI, 3, 4, true, 0>(a, Ntot, 1, 0, ev0, ev1, s);
        case 1304: return launch_gemm_one<EPI, 3, 4, true, 1>(a, Ntot, 1, 0, ev0, ev1, s);
        case 104: return launch_gemm_one<EPI, 1, 4, true, 0>(a, Ntot, 1, 0, ev0, ev1, s);
        case 1104: return launch_gemm_one<EPI, 1, 4, true, 1>(a, Ntot, 1, 0, ev0, ev1, s);
        case 1204: return launch_gemm_one<EPI, 2, 4, true, 1>(a, Ntot, 1, 0, ev0, ev1, s);
        case 1408: return launch_gemm_one<EPI, 4, 8, false, 1>(a, Ntot, 1, 0, ev0, ev1, s);
        case 808: return launch_gemm_one<EPI, 4, 8, false, 0, 4>(a, Ntot, 1, 0, ev0, ev1, s);
        case 524: return launch_gemm_one<EPI, 2, 4, true, 0, 4>(a, Ntot, 1, 0, ev0, ev1, s);
        case 1808: return launch_gemm_one<EPI, 4, 8, false, 1, 4>(a, Ntot, 1, 0, ev0, ev1, s);
        case 1404: return launch_gemm_one<EPI, 4, 4, true, 1>(a, Ntot, 1, 0, ev0, ev1, s);
    }
    return hipErrorInvalidValue;
}

bool gemm_mfma_serves(int epi, int Ntot, int K, int R) {
    (void)epi;
    return R >= GEMM_MIN_ROWS && Ntot % 16 == 0 && K % 32 == 0;
}

// Rough time of one launch in microseconds, from what was measured on the chip: a workgroup spends a fixed time per
// k-tile whatever its rows (load latency it cannot hide: 0.57 us for the narrow block alone on a compute unit, 1.17
// us per pair sharing one; 1.0 / 1.7 us for the wide block), the blocks run in rounds of 512, a split of K
// adds its summing pass, and the live rows of a block cost about 0.075 us each (x rows fetched, epilogue rows).
float gemm_mfma_estimate_us(int Ntot, int K, int R, size_t ws_bytes, bool q8) {
    const int m_blocks = (R + 127) / 128, KT = K / 32;
    const float rows_us = 0.075f * std::min(R, 128);
    if (((Ntot + 255) / 256) * m_blocks > 256) {
        const int wgs = ((Ntot + 255) / 256) * m_blocks;
        // (up to 64 rows the lower blocks serve these matrices too: measured 1.55 us per k-tile on the LM heads)
        return 3.f + KT * (R <= 64 ? 1.55f : 1.7f) * ((wgs + 511) / 512) + rows_us;
    }
    const int sp = pick_ksplit(Ntot, K, R, ws_bytes, q8);
    const int wgs = ((Ntot + 127) / 128) * m_blocks * sp, stages = (KT + sp - 1) / sp;
    float per_stage = wgs <= 256 ? 0.57f : 1.17f * ((wgs + 511) / 512);
    if (R <= 96) per_stage = wgs <= 256 ? 0.50f : 1.0f * ((wgs + 511) / 512);   // the 96-row block
    if (R <= 64) per_stage = wgs <= 256 ? 0.40f : 0.62f * ((wgs + 511) / 512);  // the 64-row block
    if (R <= 32) per_stage = wgs <= 256 ? 0.33f : 0.55f * ((wgs + 511) / 512);  // the 32-row block
    return 3.f + stages * per_stage + (sp > 1 ? 8.f : 0.f) + rows_us;
}

// Host-side contract: w0 is the re-tiled matrix, Ntot % 16 == 0, K % 32 == 0, a.x holds R fp32 rows of length K
// (x_mul = 1, x_add = 0), any R >= 1; RESID writes Ntot / 16 statistics slots per row (<= ssq_stride); LOGITS writes
// one softmax partial per row and 16-column tile (n_tiles = Ntot / 16).  With
// statistics of the input (a.ssq_in) the row scales are first reduced into scale_buf (device, R floats).
// `forced` = 1000 shares of K + 100 WM + WN selects the block shape and the split (0 = automatic; 104: 32 x 128, 204: 64 x 128, 304: 96 x 128, 404:
// 128 x 128, 408: 128 x 256, 808: 256 x 256; shares need the workspace `ws`: shares x R x Ntot floats).
hipError_t launch_gemm_mfma(const GemvArgs &a0, int epi, int forced, float *scale_buf, float *ws, size_t ws_bytes,
                            hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t s) {
    GemvArgs a = a0;
    int Ntot = a.n0;
    if (epi == EPI_QKV) Ntot = (a.nq + 2 * a.nkv) * a.hd;
    if (epi == EPI_SWIGLU) Ntot = 2 * a.n0;
    if (a.R < 1 || Ntot % 16 || a.K % 32 || a.x == nullptr || a.x_mul != 1 || a.x_add != 0) return hipErrorInvalidValue;
    if (epi == EPI_RESID && Ntot / 16 > a.ssq_stride) return hipErrorInvalidValue;
    a.row_scale = nullptr;
    if (a.ssq_in != nullptr) {
        if (scale_buf == nullptr) return hipErrorInvalidValue;
        hipLaunchKernelGGL(row_scale_k, dim3((a.R + 3) / 4), dim3(256), 0, s, a.ssq_in, a.ssq_in_slots, a.ssq_stride, a.R,
                           a.K, a.eps, scale_buf);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        a.row_scale = scale_buf;
    }
    switch (epi) {
        case EPI_PLAIN: return launch_gemm_cfg<EPI_PLAIN>(a, Ntot, forced, ws, ws_bytes, ev_start, ev_stop, s);
        case EPI_QKV: return launch_gemm_cfg<EPI_QKV>(a, Ntot, forced, ws, ws_bytes, ev_start, ev_stop, s);
        case EPI_RESID: return launch_gemm_cfg<EPI_RESID>(a, Ntot, forced, ws, ws_bytes, ev_start, ev_stop, s);
        case EPI_SWIGLU: return launch_gemm_cfg<EPI_SWIGLU>(a, Ntot, forced, ws, ws_bytes, ev_start, ev_stop, s);
        case EPI_LOGITS: return launch_gemm_cfg<EPI_LOGITS>(a, Ntot, forced, ws, ws_bytes, ev_start, ev_stop, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace sd
