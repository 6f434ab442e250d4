// Argument blocks shared by the host engine and the kernels, and the launcher prototypes.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd {

enum { DT_F32 = 0, DT_BF16 = 1 };

// Per-context decoding state, all device memory.
struct State {
    int32_t *len;         // [B] committed tokens per sequence
    int32_t *prompt_len;  // [B]
    int32_t *gamma_b;     // [B] planned gamma of the current step
    int32_t *k;           // [B] tokens drafted in the current step; 0 while the sequence is still drafting
    int32_t *ctl;         // [0] speculative-step ordinal, [1] sequences still drafting, [2] arrivals of the draft
                          // sampler's workgroups, [3] draft passes sampled since the last reset
    int32_t *tokens;      // [B][max_seq]
    int32_t max_seq;
    int32_t batch;
};

// Which positions the rows of a forward pass stand for.
enum { ROWS_PREFILL = 0, ROWS_VERIFY = 1, ROWS_DRAFT_FIRST = 2, ROWS_DRAFT_NEXT = 3 };

struct RowPlan {
    int32_t mode;   // ROWS_*
    int32_t rps;    // rows per sequence (ragged: the most any sequence has)
    int32_t arg;    // PREFILL: first position; DRAFT_NEXT: draft step j (>= 2)
    int32_t ragged; // VERIFY: sequence b has gamma_b[b] + 1 rows, packed one sequence after the other;
                    // DRAFT_NEXT: one row per sequence that still drafts (k[b] == 0), in sequence order
};

struct KVCache {
    void *k, *v;                 // one layer: [n_pages][n_kv][page_tokens x hd block], element type per model dtype
    const int32_t *block_table;  // [B][pages_per_seq] logical -> physical page
    int32_t pages_per_seq, page_tokens, page_shift, n_kv, hd;
    int32_t frag;                // arrangement inside a head's block: 0 plain, 1 fragment order (kv.hpp)
};

enum { EPI_PLAIN = 0, EPI_QKV = 1, EPI_RESID = 2, EPI_SWIGLU = 3, EPI_LOGITS = 4 };

// One fused projection: y = epilogue( scale_r * (x . W^T) ).
struct GemvArgs {
    // weights: up to three row-major matrices sharing K (QKV: wq, wk, wv; SWIGLU: gate, up)
    const void *w0, *w1, *w2;
    int32_t n0, n1, n2;
    int32_t K;
    int32_t R;                // rows of x in this launch
    const float *x;           // fp32 [.][K] (already multiplied by the norm weight when normed)
    const uint16_t *xb;       // bf16 copy of x for the matrix-core path
    int64_t xb_lo;            // element offset from xb to the bf16 remainder x - bf16(x) (0: none)
    int32_t x_mul, x_add;     // logical row r reads x row r * x_mul + x_add
    const float *ssq_in;      // [row][ssq_stride] partial sums of squares of the un-normed input, or null
    int32_t ssq_in_slots, ssq_stride;
    float eps;
    const float *row_scale;   // dense-contraction kernel only: ready-made row scales [R] (null: ones)
    int32_t rpw;              // W rows per wave (wave-dot) / 16-row groups per workgroup (matrix-core)
    const int32_t *active;    // when non-null and *active == 0 the kernel does nothing (drafting has stopped)
    const float *wscale;      // 8-bit weights: one scale per packed output column, multiplied into the reduced tile (null: 16-bit weights)
    // scratch of the kernel that shares K out over workgroups (null: that kernel is not used): partial tiles
    // [KSPLIT_MAX][Ntot / 16][16][16] fp32 and one arrival counter per set of groups, zero between launches
    float *ks_part;
    uint32_t *ks_ticket;
    // ---- epilogue ----
    float *y;                 // PLAIN: [R][N]; LOGITS: logits base; QKV: q [R][nq*hd]
    int32_t y_mul, y_add, y_stride;  // LOGITS: logical row r writes row r * y_mul + y_add ...
    const int32_t *y_rows;    // ... or, when given, row y_rows[r] * y_mul + y_add (draft passes over the sequences still drafting)
    // RESID
    float *xres;              // [R][N] residual stream, read-modify-write
    const float *g_next;      // [N] weight of the norm that consumes the new residual (null -> ones)
    float *xg;                // [R][N] xres * g_next (fp32)
    uint16_t *xgb;            // same, bf16
    int64_t xgb_lo;           // offset to its remainder half (0: none)
    float *ssq_out;           // [R][ssq_stride] one slot per workgroup
    // SWIGLU / QKV second outputs
    uint16_t *yb;             // bf16 copy of y (SWIGLU act, QKV q)
    int64_t yb_lo;            // offset to its remainder half (0: none)
    // QKV
    int32_t nq, nkv, hd;
    const float *rope_cos, *rope_sin;  // [max_seq][hd/2]
    const int32_t *row_pos, *row_seq;  // [R]
    KVCache kv;
    int32_t kv_dtype;
    // LOGITS partial softmax statistics, one per (row, tile)
    float *pm;                // max logit of the tile
    double *ps;               // sum exp((l - pm) * inv_t) over the tile
    int32_t *pa;              // argmax (lowest index) of the tile
    int32_t n_tiles;          // tiles per row (stride of the three arrays)
    float inv_t;
};

// Source of a re-tiled matrix: mode EPI_PLAIN (w0, Ntot rows), EPI_SWIGLU (gate = w0, up = w1,
// Ntot = 2 * d_ffn) or EPI_QKV (wq, wk, wv; Ntot = (nq + 2 nkv) * hd).
struct RetileArgs {
    const void *w0, *w1, *w2;
    int32_t mode, Ntot, K, nq, nkv, hd;
    int32_t q8;                  // 1: int8 sources (tiles of 16 rows x 64 k) with one fp32 scale per row
    const float *s0, *s1, *s2;   // q8: the scales of w0, w1, w2
    float *scale_out;            // q8: [Ntot] scales in packed row order (may be null)
};

struct EmbedArgs {
    State st;
    RowPlan plan;
    int32_t R;
    const void *embed;  // [V][d]
    int32_t dtype, d, vocab;
    const float *g_next;
    float *x, *xg;
    uint16_t *xgb;
    int64_t xgb_lo;
    float *ssq_out;
    int32_t ssq_stride;
    int32_t *row_pos, *row_seq;
    int32_t *row_off;   // ragged plans: [batch + 1] first row of every sequence, written by the kernel
};

struct AttnArgs {
    const float *q;       // [R][nq*hd], rotated
    const uint16_t *qb;   // bf16 copy (matrix-core kernel); null forces the plain kernel
    int64_t qb_lo, ob_lo; // offsets to the remainder halves of qb / ob (0: none)
    KVCache kv;
    int32_t kv_dtype;
    int32_t R, rps, nq;     // rps: rows per sequence (with row_off: the most any sequence has)
    int32_t batch;
    const int32_t *row_off; // [batch + 1] first row of every sequence when they differ in rows (null: b * rps)
    const int32_t *row_pos, *row_seq;
    int32_t chunk;        // KV positions per workgroup
    int32_t stream_chunks; // matrix-core kernels: 1 = the chunk is streamed slab by slab through three register buffers (chunks of 256 / 512)
    int32_t n_chunks;     // grid.x
    float scale;
    float *part_m, *part_l;  // [R][nq][n_chunks]
    float *part_o;           // [R][nq][n_chunks][hd]
    uint32_t *ticket;        // [batch][n_kv] arrival counters, zero between launches; null: the partials are merged by a second kernel
    float *o;                // [R][nq*hd]
    uint16_t *ob;            // bf16 copy
    const int32_t *active;
};

// Sampling configuration shared by the sampler kernels.
struct SampleCfg {
    float temperature;   // 0 -> greedy
    float inv_t;         // 1/T, or 1 when greedy
    uint64_t seed;
    int32_t forced;      // 1: forced acceptance landscape
    const float *alpha;  // [n_alpha]
    int32_t n_alpha;
    float tau;           // <= 0: no early stop
};

struct DraftSampleArgs {
    State st;
    SampleCfg cfg;
    int32_t j;            // draft step, 1-based
    int32_t gamma_max;
    const float *logits;  // draft logits [B][gamma_max][V]
    int32_t vocab;
    const float *pm; const double *ps; const int32_t *pa;  // partials [B*gamma_max][n_tiles]
    int32_t n_tiles, tile;
    const float *pm2; const double *ps2; const int32_t *pa2;  // level 2: one per 64 tiles, [..][n2]
    int32_t n2;
    int32_t *host_pass;   // pinned host memory, or null: [0] = ctl[3] after this pass, [1] = sequences still drafting
    // per drafted token: logit of the chosen token, row max, row sum  -> [B][gamma_max]
    float *q_logit, *q_max;
    double *q_sum;
};

struct AcceptArgs {
    State st;
    SampleCfg cfg;
    int32_t gamma;        // rows per sequence in the target logits buffer = gamma + 1
    int32_t gamma_max;
    int32_t vocab;
    const float *p_logits;  // [B][gamma+1][V], or packed rows when row_off is set
    const int32_t *row_off; // [B + 1] first target row of every sequence (null: b * (gamma + 1))
    const float *pm; const double *ps; const int32_t *pa;  // target partials [B*(gamma+1)][n_tiles]
    int32_t n_tiles, tile;
    const float *pm2; const double *ps2; const int32_t *pa2;  // level 2: one per 64 tiles, [..][n2]
    int32_t n2;
    const float *q_logits;  // [B][gamma_max][V]
    const float *q_logit, *q_max; const double *q_sum;     // [B][gamma_max]
    // scratch of the accept phase
    double *row_max, *row_sum;  // [B][gamma+1] (max as double for uniform arithmetic)
    int32_t *row_arg;           // [B][gamma+1]
    int32_t *resid_row;         // [B] 0 = no residual draw needed, else row index (1-based)
    double *resid_part;         // [B][n_resid_chunks]
    int32_t n_resid_chunks;
    uint32_t *ticket;           // [B]
    int32_t *out_A, *out_y, *out_k;  // [B] device-visible result (pinned host memory)
    int32_t *A_dev, *y_dev;     // [B] device copies
};

// ---- launchers (defined next to the kernels) -----------------------------------------------------
hipError_t launch_begin_draft(const State &st, const int32_t *gamma_plan, hipStream_t s);
hipError_t launch_embed(const EmbedArgs &a, hipStream_t s);
hipError_t launch_gemv_wavedot(const GemvArgs &a, int epi, int w_dtype, hipStream_t s);
hipError_t launch_gemv_mfma(const GemvArgs &a, int epi, int forced_cfg, hipEvent_t ev_start, hipEvent_t ev_stop,
                            hipStream_t s);
bool gemv_mfma_resident_x(int K, int R, bool q8);  // 17-64 rows: the streaming kernel keeps its x fragments in registers
constexpr int KSPLIT_MAX = 4;      // most workgroups that share the K of one group
constexpr int KSPLIT_TICKETS = 256; // arrival counters (one per set of groups: at most one per compute unit)
int gemv_mfma_groups_per_wg(int epi, int Ntot, int K, int R, int forced_cfg, bool q8 = false);  // 16-row groups per workgroup
// Prompt ingestion: the dense-contraction kernel for many rows (x read as fp32 rows, a.x).
constexpr int GEMM_MIN_ROWS = 17;  // up to 16 rows the persistent weight-streaming kernel is the faster one at any shape
bool gemm_mfma_serves(int epi, int Ntot, int K, int R);
float gemm_mfma_estimate_us(int Ntot, int K, int R, size_t workspace_bytes, bool q8 = false);  // rough time of one launch
hipError_t launch_gemm_mfma(const GemvArgs &a, int epi, int forced_cfg, float *scale_buf, float *workspace,
                            size_t workspace_bytes, hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t s);
bool gemv_wavedot_uses_split(int epi, int Ntot, int K, int R, int w_dtype);
int gemv_wavedot_tile_cols(int epi, int Ntot, int K, int R, int w_dtype);
int gemv_wavedot_pick_rpw(int epi, int N, int K, int R, int w_dtype);
hipError_t launch_attention(const AttnArgs &a, int hd, hipStream_t s);
constexpr int ATT_NC_MAX = 32;  // chunks per sequence the matrix-core attention kernel can merge
int attention_mfma_chunk(int max_seq, int wanted);  // wanted: 0 = automatic, else 64 / 128 / 256 / 512
bool attention_uses_mfma(const AttnArgs &a, int hd);
hipError_t launch_draft_sample(const DraftSampleArgs &a, hipStream_t s);
hipError_t launch_accept(const AcceptArgs &a, hipStream_t s);
hipError_t launch_row_partials(const float *logits, int rows, int vocab, int tile, float inv_t, float *pm, double *ps,
                               int32_t *pa, hipStream_t s);
hipError_t launch_merge_partials(const float *pm, const double *ps, const int32_t *pa, int n1, float inv_t, float *pm2,
                                 double *ps2, int32_t *pa2, int rows, int y_mul, int y_add, const int32_t *y_rows,
                                 const int32_t *active, hipStream_t s);
hipError_t launch_gather_qstats(const float *q_logits, const int32_t *drafted, int rows, int vocab, const float *pm,
                                const double *ps, const int32_t *pa, int n_tiles, float inv_t, float *q_logit,
                                float *q_max, double *q_sum, hipStream_t s);
hipError_t launch_retile(const RetileArgs &a, void *out, hipStream_t s);
hipError_t launch_philox(uint64_t seed, const uint32_t *ctr, int n, uint32_t *out, hipStream_t s);
hipError_t launch_fill_uniform(void *dst, int64_t n, int dtype, uint64_t seed, hipStream_t s);
hipError_t launch_kv_write(const KVCache &kv, int kv_dtype, int seq, int pos0, int n, const float *k, const float *v,
                           hipStream_t s);
hipError_t launch_copy(const void *src, void *dst, int64_t bytes, hipStream_t s);
hipError_t launch_cast_to_bf16(const float *src, uint16_t *dst, int64_t lo_off, int64_t n, hipStream_t s);
hipError_t launch_cast_to_f32(const void *src, int dtype, float *dst, int64_t n, hipStream_t s);

}  // namespace sd
