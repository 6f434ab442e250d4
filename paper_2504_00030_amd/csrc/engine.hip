// Host engine behind the C ABI of include/spec.h and include/spec_debug.h: owns the paged KV caches, the re-tiled weights (16-bit, or
// 8-bit with per-row scales), the activation and logits buffers and the HIP graphs (one per draft pass index,
// one per verification length), and strings the kernels into the three phases of a speculative step (Background
// section): gamma draft decode steps, one target verification pass over gamma+1 rows, and the accept / resample
// step.  Per projection it picks the weight-streaming or the dense-contraction kernel from measured time
// estimates (launch_proj).
#include "spec.h"
#include "spec_debug.h"
#include "gammatune.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <chrono>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "kernels/params.hpp"

using namespace sd;

namespace {

constexpr int SSQ_STRIDE = 512;
constexpr int ATT_CHUNK = 64;
constexpr int RESID_CHUNKS = 64;
constexpr int PREFILL_ROWS = 32;        // rows per sequence of one ingestion launch on the weight-streaming kernels
constexpr int PREFILL_GEMM_ROWS = 1024;  // rows (all sequences) of one ingestion launch on the dense-contraction kernels

struct ModelRT {
    spec_shape s{};
    std::vector<const void *> wq, wk, wv, wo, wg, wu, wd;
    std::vector<float *> attn_norm, ffn_norm;
    float *final_norm = nullptr;
    const void *embed = nullptr, *lm_head = nullptr;
    // re-tiled bf16 copies for the matrix-core path (empty when unused)
    std::vector<void *> t_qkv, t_wo, t_gu, t_wd;
    void *t_lm = nullptr;
    bool mfma_ok = false;
    int Rmax = 0;
    size_t gemm_ws_bytes = 0;
    int32_t *row_off = nullptr;                        // [batch + 1] first row of every sequence of a ragged pass
    bool q8 = false;                                   // projection matrices and LM head are 8-bit
    std::vector<float *> sc_qkv, sc_wo, sc_gu, sc_wd;  // their scales in packed row order (null entries otherwise)
    float *sc_lm = nullptr;
    float *x = nullptr, *xg = nullptr, *ssq = nullptr, *row_scale = nullptr, *gemm_ws = nullptr, *q = nullptr, *ao = nullptr, *act = nullptr;
    float *ks_part = nullptr;       // partial tiles of the projections whose K is shared out over workgroups
    uint32_t *ks_ticket = nullptr;  // their arrival counters
    uint16_t *xgb = nullptr, *qb = nullptr, *aob = nullptr, *actb = nullptr;
    int32_t *row_pos = nullptr, *row_seq = nullptr;
    std::vector<void *> kpool, vpool;
    int32_t *block_table = nullptr;
    int pages_per_seq = 0, n_pages = 0;
    float *rope_cos = nullptr, *rope_sin = nullptr;
    float *part_m = nullptr, *part_l = nullptr, *part_o = nullptr;
    uint32_t *att_ticket = nullptr;  // [B][n_kv_heads] arrival counters of the attention chunks (zero between launches)
    int n_chunks = 0;
    // logits and their tile partials
    float *logits = nullptr;
    int logit_rows = 0;
    float *pm = nullptr, *pm2 = nullptr;
    double *ps = nullptr, *ps2 = nullptr;
    int32_t *pa = nullptr, *pa2 = nullptr;
    int tiles_cap = 0, tiles2_cap = 0;
};

}  // namespace

struct spec_ctx {
    spec_config cfg{};
    hipStream_t stream = nullptr;
    bool own_stream = false;
    hipStream_t side_stream = nullptr;  // second stream of the same (default) priority: the draft model's prompt ingestion
    ModelRT tgt, drf;
    State st{};
    std::vector<void *> dev_allocs, host_allocs;
    int64_t dev_bytes = 0;
    std::string err;
    // host mirrors
    std::vector<int32_t> h_len;
    int32_t *h_gamma_plan = nullptr;  // pinned, read by the device
    int32_t *h_out = nullptr;         // pinned [3][B]: A, y, k
    int32_t *h_pass = nullptr, *d_pass = nullptr;  // pinned [2]: draft passes sampled, sequences still drafting
    int32_t passes_launched = 0;      // draft sample kernels enqueued since the last reset of ctl[3]
    int32_t *d_gamma_plan = nullptr, *d_out = nullptr;
    // sampling
    SampleCfg scfg{};
    float *d_alpha = nullptr;
    int n_alpha = 0;
    float *q_logit = nullptr, *q_max = nullptr;
    double *q_sum = nullptr;
    double *row_max = nullptr, *row_sum = nullptr, *resid_part = nullptr;
    int32_t *row_arg = nullptr, *resid_row = nullptr, *A_dev = nullptr, *y_dev = nullptr;
    uint32_t *ticket = nullptr;
    // logits tiling of the last launches
    int d_tile = 0, d_ntiles = 0, t_tile = 0, t_ntiles = 0;
    // state machine: 0 = created, 1 = ready to draft, 2 = drafted, 3 = verified
    int phase = 0;
    int cur_gamma = 0;
    int verify_only_rows = 0;  // rows of the last spec_debug_verify_rows pass (0: the last target pass was a step's)
    int cur_rows = 0;      // rows of the current step's verification pass when it is ragged, else 0
    bool ragged_ok = false;  // several sequences and a target whose attention takes ragged rows
    bool compact_ok = false; // the same for the draft model: passes after the first hold only the sequences still drafting
    bool prefilled = false;
    std::map<int, hipGraphExec_t> g_draft, g_pass;  // whole draft phase per gamma, draft pass j
    // verification pass per (gamma, rows), with the logits tiling its LM-head launch uses: the accept kernels run
    // outside the graph and must index the softmax partials the way the replayed graph writes them
    struct VerifyGraph { hipGraphExec_t exec; int tile, ntiles; };
    std::map<int, VerifyGraph> g_verify;
    std::vector<hipGraph_t> graphs;
    // optional timing of one kernel class with event pairs (direct launches only)
    // timed kernel class (-1: none, 0: every class of both models) and model; classes: 1 QKV, 2 output and down
    // projection together, 3 gate/up, 4 LM head, 5 output projection, 6 down projection, 7 attention with its merge
    int prof_epi = -1, prof_model = 0;
    std::vector<int> prof_tag;            // per event pair: 16 * model + class
    bool capturing = false;
    std::vector<hipEvent_t> prof_events;  // start, stop, start, stop, ...
    size_t prof_used = 0;
};

namespace {

thread_local std::string g_last_err;  // failures that leave no context behind (spec_init)

int fail(spec_ctx *c, int code, const std::string &msg) {
    if (c) c->err = msg;
    g_last_err = msg;
    return code;
}

#define HIPCHK(c, call)                                                                              \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess)                                                                        \
            return fail((c), SPEC_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));          \
    } while (0)

template <typename T> int dalloc(spec_ctx *c, T **p, size_t n) {
    void *v = nullptr;
    const size_t bytes = (n ? n : 1) * sizeof(T);
    if (hipMalloc(&v, bytes) != hipSuccess) return fail(c, SPEC_ENOMEM, "hipMalloc failed");
    if (hipMemsetAsync(v, 0, bytes, c->stream) != hipSuccess) return fail(c, SPEC_EHIP, "hipMemsetAsync failed");
    c->dev_allocs.push_back(v);
    c->dev_bytes += (int64_t)bytes;
    *p = reinterpret_cast<T *>(v);
    return SPEC_OK;
}

// device allocation that is fully overwritten by its first use (no zero fill)
template <typename T> int dalloc_raw(spec_ctx *c, T **p, size_t n) {
    void *v = nullptr;
    const size_t bytes = (n ? n : 1) * sizeof(T);
    if (hipMalloc(&v, bytes) != hipSuccess) return fail(c, SPEC_ENOMEM, "hipMalloc failed");
    c->dev_allocs.push_back(v);
    c->dev_bytes += (int64_t)bytes;
    *p = reinterpret_cast<T *>(v);
    return SPEC_OK;
}

#define TRY(expr)                       \
    do {                                \
        int rc_ = (expr);               \
        if (rc_ != SPEC_OK) return rc_; \
    } while (0)

int check_shape(spec_ctx *c, const spec_shape &s, const char *who) {
    auto bad = [&](const char *m) { return fail(c, SPEC_EINVAL, std::string(who) + ": " + m); };
    if (s.n_layers < 1 || s.d_model < 8 || s.n_q_heads < 1 || s.n_kv_heads < 1 || s.head_dim < 8 || s.d_ffn < 8 ||
        s.vocab < 2)
        return bad("non-positive dimension");
    if (s.n_q_heads % s.n_kv_heads) return bad("n_q_heads not a multiple of n_kv_heads");
    if (s.head_dim % 8) return bad("head_dim must be a multiple of 8");
    if (s.dtype != SPEC_F32 && s.dtype != SPEC_BF16 && s.dtype != SPEC_Q8) return bad("unknown dtype");
    if (s.dtype == SPEC_Q8) {
        if (s.d_model % 64 || s.d_ffn % 64 || (s.n_q_heads * s.head_dim) % 64 || s.vocab % 16 || (s.head_dim / 2) % 8)
            return bad("8-bit weights need d_model, n_q_heads * head_dim, d_ffn multiples of 64, vocab of 16, head_dim of 16");
        if (c->cfg.gemv_path == SPEC_PATH_WAVEDOT) return bad("8-bit weights run on the matrix-core kernels only");
    }
    const int vec = s.dtype == SPEC_F32 ? 4 : 8;
    if (s.d_model % vec || s.d_ffn % vec || (s.n_q_heads * s.head_dim) % vec) return bad("row length not 16-byte aligned");
    if (s.d_ffn % 2) return bad("d_ffn must be even");
    if (!(s.rms_eps > 0.f) || !(s.rope_theta > 0.f)) return bad("bad rms_eps / rope_theta");
    for (int R = 1; R <= 4; ++R) {
        const int cols = gemv_wavedot_tile_cols(EPI_RESID, s.d_model, s.d_ffn, R, s.dtype == SPEC_F32 ? SPEC_F32 : SPEC_BF16);
        if ((s.d_model + cols - 1) / cols > SSQ_STRIDE) return bad("d_model too large");
    }
    return SPEC_OK;
}

int check_weights(spec_ctx *c, const spec_shape &s, const spec_weights *w, const char *who) {
    auto bad = [&](const char *m) { return fail(c, SPEC_EINVAL, std::string(who) + ": " + m); };
    if (!w || !w->tok_embed || !w->lm_head || !w->final_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate ||
        !w->w_up || !w->w_down || !w->attn_norm || !w->ffn_norm)
        return bad("null weight pointer");
    for (int l = 0; l < s.n_layers; ++l) {
        const void *ps[] = {w->wq[l], w->wk[l], w->wv[l], w->wo[l], w->w_gate[l], w->w_up[l], w->w_down[l],
                            w->attn_norm[l], w->ffn_norm[l]};
        for (const void *p : ps) {
            if (!p) return bad("null layer weight");
            if (reinterpret_cast<uintptr_t>(p) % 16) return bad("weight not 16-byte aligned");
        }
    }
    if (s.dtype == SPEC_Q8) {
        if (!w->wq_scale || !w->wk_scale || !w->wv_scale || !w->wo_scale || !w->w_gate_scale || !w->w_up_scale ||
            !w->w_down_scale || !w->lm_head_scale)
            return bad("8-bit weights without scales");
        for (int l = 0; l < s.n_layers; ++l) {
            const void *ps[] = {w->wq_scale[l], w->wk_scale[l], w->wv_scale[l], w->wo_scale[l], w->w_gate_scale[l],
                                w->w_up_scale[l], w->w_down_scale[l]};
            for (const void *p : ps)
                if (!p) return bad("null layer scale");
        }
        if (w->lm_head == w->tok_embed) return bad("8-bit LM head cannot alias the bf16 embedding");
    }
    return SPEC_OK;
}

// Whether the projections of a model run on the matrix-core kernels (re-tiled bf16 weights).
bool model_on_matrix_cores(const spec_config &g, const spec_shape &s) {
    const int d = s.d_model, qd = s.n_q_heads * s.head_dim;
    if (s.dtype == SPEC_Q8) return true;  // check_shape admits no other 8-bit model
    return s.dtype == SPEC_BF16 && g.gemv_path != SPEC_PATH_WAVEDOT && d % 32 == 0 && qd % 32 == 0 && s.d_ffn % 32 == 0 &&
           s.vocab % 16 == 0 && (s.head_dim / 2) % 8 == 0 && d % 16 == 0;
}

// Rows of one prompt-ingestion launch (all sequences together).  A model on the matrix cores whose attention
// also runs on them ingests through the dense-contraction kernels, PREFILL_GEMM_ROWS rows at a time; otherwise
// PREFILL_ROWS per sequence (the plain attention kernel holds at most 128 rows of a sequence).
// Whether the attention of a model on the matrix cores runs on the matrix-core attention kernels as well.
bool attention_on_matrix_cores(const spec_config &g, const spec_shape &s) {
    const int hd = s.head_dim;
    const int chunk = attention_mfma_chunk(g.max_seq, g.attn_chunk);
    return g.page_tokens % 4 == 0 && (hd == 32 || hd == 64 || hd == 128) && (g.max_seq + chunk - 1) / chunk <= ATT_NC_MAX;
}

int ingest_rows(const spec_config &g, const spec_shape &s) {
    const bool attn_mc = attention_on_matrix_cores(g, s);
    if (model_on_matrix_cores(g, s) && attn_mc && s.d_model / 16 <= SSQ_STRIDE) return std::max(PREFILL_GEMM_ROWS, g.batch);
    return std::min(128, g.batch * PREFILL_ROWS);
}

int build_model(spec_ctx *c, ModelRT &m, const spec_shape &s, const spec_weights *w, int Rmax, int logit_rows) {
    m.s = s;
    m.q8 = s.dtype == SPEC_Q8;
    if (m.q8) m.s.dtype = SPEC_BF16;  // from here on dtype is the storage type of embedding, norms and KV cache
    m.Rmax = Rmax;
    const int L = s.n_layers, d = s.d_model, qd = s.n_q_heads * s.head_dim;
    const hipStream_t st = c->stream;
    for (int l = 0; l < L; ++l) {
        m.wq.push_back(w->wq[l]); m.wk.push_back(w->wk[l]); m.wv.push_back(w->wv[l]); m.wo.push_back(w->wo[l]);
        m.wg.push_back(w->w_gate[l]); m.wu.push_back(w->w_up[l]); m.wd.push_back(w->w_down[l]);
        float *a = nullptr, *f = nullptr;
        TRY(dalloc(c, &a, d));
        TRY(dalloc(c, &f, d));
        HIPCHK(c, launch_cast_to_f32(w->attn_norm[l], m.s.dtype, a, d, st));
        HIPCHK(c, launch_cast_to_f32(w->ffn_norm[l], m.s.dtype, f, d, st));
        m.attn_norm.push_back(a);
        m.ffn_norm.push_back(f);
    }
    TRY(dalloc(c, &m.final_norm, d));
    HIPCHK(c, launch_cast_to_f32(w->final_norm, m.s.dtype, m.final_norm, d, st));
    m.embed = w->tok_embed;
    m.lm_head = w->lm_head;

    // re-tiled copies for the matrix-core kernels
    const int kvd = s.n_kv_heads * s.head_dim;
    m.mfma_ok = model_on_matrix_cores(c->cfg, s);
    if (m.mfma_ok) {
        // 8-bit weights: the tiled copy holds N*K bytes and comes with the scales in packed row order
        auto retile = [&](int mode, const void *w0, const void *w1, const void *w2, const void *s0, const void *s1,
                          const void *s2, int Ntot, int K, void **out, float **scale_out) {
            uint8_t *buf = nullptr;
            TRY(dalloc_raw(c, &buf, (size_t)Ntot * K * (m.q8 ? 1 : 2)));
            RetileArgs ra{};
            ra.w0 = w0; ra.w1 = w1; ra.w2 = w2; ra.mode = mode; ra.Ntot = Ntot; ra.K = K;
            ra.nq = s.n_q_heads; ra.nkv = s.n_kv_heads; ra.hd = s.head_dim;
            *scale_out = nullptr;
            if (m.q8) {
                float *sc = nullptr;
                TRY(dalloc(c, &sc, (size_t)Ntot));
                ra.q8 = 1; ra.scale_out = sc;
                ra.s0 = reinterpret_cast<const float *>(s0); ra.s1 = reinterpret_cast<const float *>(s1);
                ra.s2 = reinterpret_cast<const float *>(s2);
                *scale_out = sc;
            }
            HIPCHK(c, launch_retile(ra, buf, st));
            *out = buf;
            return (int)SPEC_OK;
        };
        for (int l = 0; l < L; ++l) {
            void *t = nullptr;
            float *sc = nullptr;
            const bool q = m.q8;
            TRY(retile(EPI_QKV, w->wq[l], w->wk[l], w->wv[l], q ? w->wq_scale[l] : nullptr, q ? w->wk_scale[l] : nullptr,
                       q ? w->wv_scale[l] : nullptr, qd + 2 * kvd, d, &t, &sc));
            m.t_qkv.push_back(t); m.sc_qkv.push_back(sc);
            TRY(retile(EPI_PLAIN, w->wo[l], nullptr, nullptr, q ? w->wo_scale[l] : nullptr, nullptr, nullptr, d, qd, &t, &sc));
            m.t_wo.push_back(t); m.sc_wo.push_back(sc);
            TRY(retile(EPI_SWIGLU, w->w_gate[l], w->w_up[l], nullptr, q ? w->w_gate_scale[l] : nullptr,
                       q ? w->w_up_scale[l] : nullptr, nullptr, 2 * s.d_ffn, d, &t, &sc));
            m.t_gu.push_back(t); m.sc_gu.push_back(sc);
            TRY(retile(EPI_PLAIN, w->w_down[l], nullptr, nullptr, q ? w->w_down_scale[l] : nullptr, nullptr, nullptr, d, s.d_ffn,
                       &t, &sc));
            m.t_wd.push_back(t); m.sc_wd.push_back(sc);
        }
        TRY(retile(EPI_PLAIN, w->lm_head, nullptr, nullptr, m.q8 ? w->lm_head_scale : nullptr, nullptr, nullptr, s.vocab, d,
                   &m.t_lm, &m.sc_lm));
    }

    const size_t R = (size_t)Rmax;
    TRY(dalloc(c, &m.x, R * d));
    TRY(dalloc(c, &m.xg, R * d));
    TRY(dalloc(c, &m.xgb, 2 * R * d));  // hi half, then the remainder half
    TRY(dalloc(c, &m.ssq, R * SSQ_STRIDE));
    TRY(dalloc(c, &m.row_scale, R));
    if (m.mfma_ok) {
        // partial results of projections whose k-tiles are shared out over workgroups: the matrices with few
        // output columns (d_model, QKV) at up to 512 rows, eight shares
        m.gemm_ws_bytes = (size_t)8 * std::min<size_t>(R, 512) * std::max(d, qd + 2 * kvd) * sizeof(float);
        TRY(dalloc(c, &m.gemm_ws, m.gemm_ws_bytes / sizeof(float)));
    }
    if (m.mfma_ok) {
        const int n_max = std::max(std::max(d, qd + 2 * kvd), std::max(2 * s.d_ffn, s.vocab));
        TRY(dalloc(c, &m.ks_part, (size_t)KSPLIT_MAX * ((n_max + 15) / 16) * 256));
        TRY(dalloc(c, &m.ks_ticket, (size_t)KSPLIT_TICKETS));
    }
    TRY(dalloc(c, &m.q, R * qd));
    TRY(dalloc(c, &m.qb, 2 * R * qd));
    TRY(dalloc(c, &m.ao, R * qd));
    TRY(dalloc(c, &m.aob, 2 * R * qd));
    TRY(dalloc(c, &m.act, R * s.d_ffn));
    TRY(dalloc(c, &m.actb, 2 * R * s.d_ffn));
    TRY(dalloc(c, &m.row_pos, R));
    TRY(dalloc(c, &m.row_seq, R));
    TRY(dalloc(c, &m.row_off, (size_t)c->cfg.batch + 1));

    // paged KV cache: sequence-interleaved physical pages by default
    const int PT = c->cfg.page_tokens;
    m.pages_per_seq = (c->cfg.max_seq + PT - 1) / PT;
    m.n_pages = m.pages_per_seq * c->cfg.batch;
    const size_t esz = m.s.dtype == SPEC_BF16 ? 2 : 4;
    const size_t pool = (size_t)m.n_pages * s.n_kv_heads * PT * s.head_dim * esz;
    for (int l = 0; l < L; ++l) {
        uint8_t *k = nullptr, *v = nullptr;
        TRY(dalloc(c, &k, pool));
        TRY(dalloc(c, &v, pool));
        m.kpool.push_back(k);
        m.vpool.push_back(v);
    }
    TRY(dalloc(c, &m.block_table, (size_t)m.n_pages));
    std::vector<int32_t> bt((size_t)m.n_pages);
    for (int b = 0; b < c->cfg.batch; ++b)
        for (int p = 0; p < m.pages_per_seq; ++p) bt[(size_t)b * m.pages_per_seq + p] = p * c->cfg.batch + b;
    HIPCHK(c, hipStreamSynchronize(c->stream));  // the zero fills above run on the context's stream
    HIPCHK(c, hipMemcpy(m.block_table, bt.data(), bt.size() * sizeof(int32_t), hipMemcpyHostToDevice));

    // rotary tables, angles in double
    const int half = s.head_dim / 2;
    std::vector<float> cs((size_t)c->cfg.max_seq * half), sn(cs.size());
    for (int p = 0; p < c->cfg.max_seq; ++p)
        for (int j = 0; j < half; ++j) {
            const double ang = (double)p * std::pow((double)s.rope_theta, -2.0 * j / s.head_dim);
            cs[(size_t)p * half + j] = (float)std::cos(ang);
            sn[(size_t)p * half + j] = (float)std::sin(ang);
        }
    TRY(dalloc(c, &m.rope_cos, cs.size()));
    TRY(dalloc(c, &m.rope_sin, sn.size()));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(m.rope_cos, cs.data(), cs.size() * sizeof(float), hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(m.rope_sin, sn.data(), sn.size() * sizeof(float), hipMemcpyHostToDevice));

    m.n_chunks = (c->cfg.max_seq + ATT_CHUNK - 1) / ATT_CHUNK;
    const size_t pn = R * s.n_q_heads * m.n_chunks;
    TRY(dalloc(c, &m.part_m, pn));
    TRY(dalloc(c, &m.part_l, pn));
    TRY(dalloc(c, &m.part_o, pn * s.head_dim));
    TRY(dalloc(c, &m.att_ticket, (size_t)c->cfg.batch * s.n_kv_heads));

    m.logit_rows = logit_rows;
    TRY(dalloc(c, &m.logits, (size_t)logit_rows * s.vocab));
    m.tiles_cap = (s.vocab + 15) / 16 + 1;  // the finest tiling any logits kernel uses is 16 columns
    TRY(dalloc(c, &m.pm, (size_t)logit_rows * m.tiles_cap));
    TRY(dalloc(c, &m.ps, (size_t)logit_rows * m.tiles_cap));
    TRY(dalloc(c, &m.pa, (size_t)logit_rows * m.tiles_cap));
    m.tiles2_cap = (m.tiles_cap + 63) / 64;
    TRY(dalloc(c, &m.pm2, (size_t)logit_rows * m.tiles2_cap));
    TRY(dalloc(c, &m.ps2, (size_t)logit_rows * m.tiles2_cap));
    TRY(dalloc(c, &m.pa2, (size_t)logit_rows * m.tiles2_cap));
    return SPEC_OK;
}

KVCache kv_of(const spec_ctx *c, const ModelRT &m, int l) {
    KVCache kv;
    kv.k = m.kpool[l];
    kv.v = m.vpool[l];
    kv.block_table = m.block_table;
    kv.pages_per_seq = m.pages_per_seq;
    kv.page_tokens = c->cfg.page_tokens;
    int sh = 0;
    while ((1 << sh) < c->cfg.page_tokens) ++sh;
    kv.page_shift = sh;
    kv.n_kv = m.s.n_kv_heads;
    kv.hd = m.s.head_dim;
    kv.frag = m.s.head_dim % 32 == 0 && c->cfg.page_tokens >= 16 ? 1 : 0;
    return kv;
}

// Event pair around the launches of one kernel class.  With `in_dispatch` the launcher hands the pair to
// the dispatch itself (kernel start / end); otherwise the pair is recorded on the stream around the launch.
struct ProfScope {
    spec_ctx *c;
    bool on, in_dispatch;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    ProfScope(spec_ctx *c_, const ModelRT &m, int cls, bool in_dispatch_) : c(c_), on(false), in_dispatch(in_dispatch_) {
        if (c->prof_epi < 0 || c->capturing) return;
        const int model = &m == &c->tgt ? 1 : 0;
        if (c->prof_epi != 0) {
            const bool hit = c->prof_epi == cls || (c->prof_epi == 2 && (cls == 5 || cls == 6));
            if (!hit || c->prof_model != model) return;
        }
        if (c->prof_used + 2 > c->prof_events.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
            c->prof_events.push_back(a);
            c->prof_events.push_back(b);
            c->prof_tag.push_back(0);
        }
        c->prof_tag[c->prof_used / 2] = 16 * model + cls;
        on = in_dispatch || hipEventRecord(c->prof_events[c->prof_used], c->stream) == hipSuccess;
        if (on && in_dispatch) { ev0 = c->prof_events[c->prof_used]; ev1 = c->prof_events[c->prof_used + 1]; }
    }
    ~ProfScope() {
        if (!on) return;
        if (!in_dispatch) (void)hipEventRecord(c->prof_events[c->prof_used + 1], c->stream);
        c->prof_used += 2;
    }
};

constexpr int MFMA_MIN_ROWS = 1;  // measured: the matrix-core kernel streams faster than wave dot products at every row count

bool use_mfma(const spec_ctx *c, const ModelRT &m, int R) {
    if (!m.mfma_ok) return false;
    return c->cfg.gemv_path == SPEC_PATH_MFMA || R >= MFMA_MIN_ROWS;
}

// Launch one fused projection on whichever kernel family serves R rows; `tiled` is the re-tiled
// copy of the same matrices.  Returns the number of workgroups through *blocks.
int launch_proj(spec_ctx *c, ModelRT &m, GemvArgs a, int epi, const void *tiled, int Ntot, int *blocks,
                int *tile_cols, int prof_class = 0) {
    ProfScope ps_(c, m, prof_class ? prof_class : epi, use_mfma(c, m, a.R));
    // Many rows (prompt ingestion, verification of a batch): the dense-contraction kernel.  Its time hardly depends
    // on the row count.  The weight-streaming kernel beyond the 16 rows of its persistent form is bound by what a
    // compute unit fetches: per 16-row group of W its 32 K bytes (16 K with 8-bit weights) plus the 4 K bytes of
    // each row of x, shared by the groups of a workgroup, at about 38 GB/s per compute unit (measured on the 8B and
    // 1B shapes at 17-128 rows: this model and the dense estimate pick the faster kernel to within 0.5 % of the
    // summed times).  Whichever estimate is lower runs; beyond 128 rows the dense kernel is the only one.
    bool dense = m.mfma_ok && gemm_mfma_serves(epi, Ntot, a.K, a.R) && a.x_mul == 1 && a.x_add == 0;
    if (dense && a.R <= 128) {
        const int ng = gemv_mfma_groups_per_wg(epi, Ntot, a.K, a.R, 0, m.q8);
        const double groups_per_cu = std::max(1.0, Ntot / 16 / 256.0);
        // with the x fragments resident (short K, up to 64 rows) only the weights stream, at what a compute unit
        // fetches in the persistent kernels (about 23 GB/s)
        const double stream_us = gemv_mfma_resident_x(a.K, a.R, m.q8)
                                     ? 2.5 + groups_per_cu * a.K * 32.0 / 23e3
                                     : 2.5 + groups_per_cu * a.K * ((m.q8 ? 16.0 : 32.0) + 4.0 * a.R / ng) / 38e3;
        dense = gemm_mfma_estimate_us(Ntot, a.K, a.R, m.gemm_ws_bytes, m.q8) < stream_us;
    }
    if (dense) {
        // statistics slots and softmax partials are per 16-row group of W
        a.w0 = tiled; a.w1 = a.w2 = nullptr;
        if (epi == EPI_LOGITS) a.n_tiles = Ntot / 16;
        if (blocks) *blocks = Ntot / 16;
        if (tile_cols) *tile_cols = 16;
        if (epi == EPI_LOGITS && Ntot / 16 > m.tiles_cap) return fail(c, SPEC_EINVAL, "logits tiling exceeds the partial buffers");
        if (epi == EPI_RESID && Ntot / 16 > SSQ_STRIDE) return fail(c, SPEC_EINVAL, "too many statistics slots");
        HIPCHK(c, launch_gemm_mfma(a, epi, 0, m.row_scale, m.gemm_ws, m.gemm_ws_bytes, ps_.ev0, ps_.ev1, c->stream));
        return SPEC_OK;
    }
    if (use_mfma(c, m, a.R)) {
        a.w0 = tiled; a.w1 = a.w2 = nullptr;
        const int ng = gemv_mfma_groups_per_wg(epi, Ntot, a.K, a.R, 0, m.q8);
        const int nb = (Ntot / 16 + ng - 1) / ng;
        if (epi == EPI_LOGITS) a.n_tiles = nb;
        if (blocks) *blocks = nb;
        if (tile_cols) *tile_cols = 16 * ng;
        if (epi == EPI_LOGITS && nb > m.tiles_cap) return fail(c, SPEC_EINVAL, "logits tiling exceeds the partial buffers");
        if (epi == EPI_RESID && nb > SSQ_STRIDE) return fail(c, SPEC_EINVAL, "too many statistics slots");
        HIPCHK(c, launch_gemv_mfma(a, epi, 0, ps_.ev0, ps_.ev1, c->stream));
        return SPEC_OK;
    }
    const bool split = gemv_wavedot_uses_split(epi, Ntot, a.K, a.R, m.s.dtype);
    const int cols = gemv_wavedot_tile_cols(epi, Ntot, a.K, a.R, m.s.dtype);
    a.rpw = split ? 0 : gemv_wavedot_pick_rpw(epi, Ntot, a.K, a.R, m.s.dtype);
    const int nb = (Ntot + cols - 1) / cols;
    if (epi == EPI_LOGITS) a.n_tiles = nb;
    if (blocks) *blocks = nb;
    if (tile_cols) *tile_cols = cols;
    if (epi == EPI_RESID && nb > SSQ_STRIDE) return fail(c, SPEC_EINVAL, "too many statistics slots");
    if (epi == EPI_LOGITS && nb > m.tiles_cap) return fail(c, SPEC_EINVAL, "logits tiling exceeds the partial buffers");
    HIPCHK(c, launch_gemv_wavedot(a, epi, m.s.dtype, c->stream));
    return SPEC_OK;
}

struct LogitsPlan {
    bool want = false;
    int rows = 0;           // logits rows produced
    int x_mul = 1, x_add = 0;
    int y_mul = 1, y_add = 0;
    const int32_t *y_rows = nullptr;  // device: output row of every logical row (null: the row itself)
    int *tile = nullptr, *ntiles = nullptr;
};

// Enqueue one forward pass of model m over R = batch * plan.rps rows.
// `rows_total`: rows of a ragged plan (sequence b has its planned gamma + 1 of them), else 0.
int forward(spec_ctx *c, ModelRT &m, const RowPlan &plan, const LogitsPlan &lp, bool draft_phase, int rows_total = 0) {
    const spec_shape &s = m.s;
    const int B = c->cfg.batch, R = plan.ragged ? rows_total : B * plan.rps;
    const int d = s.d_model, qd = s.n_q_heads * s.head_dim, ffn = s.d_ffn;
    const hipStream_t st = c->stream;
    const int32_t *active = (draft_phase && plan.mode == ROWS_DRAFT_NEXT) ? &c->st.ctl[1] : nullptr;
    if (R > m.Rmax) return fail(c, SPEC_EINVAL, "forward: too many rows");

    EmbedArgs e{};
    e.st = c->st; e.plan = plan; e.R = R; e.embed = m.embed; e.dtype = s.dtype; e.d = d; e.vocab = s.vocab;
    // bf16 activation buffers hold a hi half and, Rmax rows later, the remainder half (matrix-core path)
    const int64_t RM = m.mfma_ok ? (int64_t)m.Rmax : 0;
    const int64_t xgb_lo = RM * s.d_model, qb_lo = RM * s.n_q_heads * s.head_dim, aob_lo = qb_lo, actb_lo = RM * s.d_ffn;
    e.g_next = m.attn_norm[0]; e.x = m.x; e.xg = m.xg; e.xgb = m.xgb; e.xgb_lo = xgb_lo; e.ssq_out = m.ssq; e.ssq_stride = SSQ_STRIDE;
    e.row_pos = m.row_pos; e.row_seq = m.row_seq; e.row_off = m.row_off;
    HIPCHK(c, launch_embed(e, st));
    int slots = 1;

    auto base = [&](int K, const float *x, const uint16_t *xb, int64_t xb_lo) {
        GemvArgs a{};
        a.K = K; a.R = R; a.x = x; a.xb = xb; a.xb_lo = xb_lo; a.x_mul = 1; a.x_add = 0; a.eps = s.rms_eps; a.active = active;
        a.ks_part = m.ks_part; a.ks_ticket = m.ks_ticket;
        a.ssq_stride = SSQ_STRIDE;
        return a;
    };
    const int kvd = s.n_kv_heads * s.head_dim;
    const bool tiled = m.mfma_ok;
    for (int l = 0; l < s.n_layers; ++l) {
        {   // fused QKV projection + RoPE + KV write
            GemvArgs a = base(d, m.xg, m.xgb, xgb_lo);
            a.w0 = m.wq[l]; a.w1 = m.wk[l]; a.w2 = m.wv[l];
            a.n0 = qd; a.n1 = a.n2 = kvd;
            a.ssq_in = m.ssq; a.ssq_in_slots = slots;
            a.y = m.q; a.yb = m.qb; a.yb_lo = qb_lo; a.nq = s.n_q_heads; a.nkv = s.n_kv_heads; a.hd = s.head_dim;
            a.rope_cos = m.rope_cos; a.rope_sin = m.rope_sin; a.row_pos = m.row_pos; a.row_seq = m.row_seq;
            a.kv = kv_of(c, m, l); a.kv_dtype = s.dtype;
            a.wscale = tiled ? m.sc_qkv[l] : nullptr;
            TRY(launch_proj(c, m, a, EPI_QKV, tiled ? m.t_qkv[l] : nullptr, qd + 2 * kvd, nullptr, nullptr));
        }
        {
            AttnArgs t{};
            t.q = m.q; t.qb = c->cfg.gemv_path == SPEC_PATH_WAVEDOT ? nullptr : m.qb; t.kv = kv_of(c, m, l); t.kv_dtype = s.dtype; t.R = R; t.rps = plan.rps; t.nq = s.n_q_heads; t.batch = B; t.row_off = plan.ragged ? m.row_off : nullptr;
            t.row_pos = m.row_pos; t.row_seq = m.row_seq; t.chunk = ATT_CHUNK; t.n_chunks = m.n_chunks;
            t.scale = 1.0f / std::sqrt((float)s.head_dim);
            t.part_m = m.part_m; t.part_l = m.part_l; t.part_o = m.part_o; t.ticket = m.att_ticket; t.o = m.ao; t.ob = m.aob; t.active = active;
            t.qb_lo = qb_lo; t.ob_lo = aob_lo;
            if (attention_uses_mfma(t, s.head_dim)) {
                // long row runs (prompt ingestion) take the largest chunk: their cost is the traffic of the chunk
                // partials, one per (row, head, chunk), not the latency of a chunk
                int wanted = plan.rps >= 64 && c->cfg.attn_chunk == 0 ? 256 : c->cfg.attn_chunk;
                // Decode and verification rows (not prompt ingestion) stream a long chunk through three register
                // buffers instead of holding a short one whole (i) where the capacity makes the chunks 512 positions long
                // (more than 4096 positions per sequence) or a chunk of 256 / 512 is asked for, and (ii) where the
                // automatic chunks would make more than 1024 workgroups of the launch and the capacity is at least two
                // long chunks: then 512-position chunks are taken in their place.  Measured, 13B-shaped verification of
                // one row per sequence at 4096 cached positions: 6.40 -> 5.99 ms for one sequence, 13.2 -> 10.3 ms for
                // eight; at 2048 positions and eight sequences 8.44 -> 8.08 ms; 8B-shaped pair, 16 / 32 sequences: +6 % /
                // +3 % tokens/s.  Not taken: streaming automatic 256-position chunks of a single sequence (2 % slower),
                // and long chunks when the capacity is one of them (eight sequences at 512 positions: 3 % slower).
                static const bool no_stream = std::getenv("SPEC_NO_ATTN_STREAM") != nullptr;
                bool stream = false;
                if (plan.mode != ROWS_PREFILL && plan.rps < 64 && !no_stream && c->cfg.page_tokens >= 16) {
                    const int auto_chunk = attention_mfma_chunk(c->cfg.max_seq, wanted);
                    stream = auto_chunk >= 512 || wanted == 256;
                    if (wanted == 0 && c->cfg.max_seq >= 1024 &&
                        (int64_t)B * s.n_kv_heads * ((c->cfg.max_seq + auto_chunk - 1) / auto_chunk) > 1024) {
                        wanted = 512;
                        stream = true;
                    }
                }
                const int chunk = attention_mfma_chunk(c->cfg.max_seq, wanted);
                const int nch = (c->cfg.max_seq + chunk - 1) / chunk;
                if (nch <= ATT_NC_MAX) { t.chunk = chunk; t.n_chunks = nch; t.stream_chunks = stream && chunk >= 256 && chunk <= 512; }
                else t.qb = nullptr;  // capacity beyond the merge of the matrix-core kernel: plain kernel
            }
            ProfScope ps_(c, m, 7, false);  // events on the stream around both launches (attention and its merge)
            HIPCHK(c, launch_attention(t, s.head_dim, st));
        }
        {   // output projection + residual
            GemvArgs a = base(qd, m.ao, m.aob, aob_lo);
            a.w0 = m.wo[l]; a.n0 = d;
            a.xres = m.x; a.g_next = m.ffn_norm[l]; a.xg = m.xg; a.xgb = m.xgb; a.xgb_lo = xgb_lo; a.ssq_out = m.ssq;
            a.wscale = tiled ? m.sc_wo[l] : nullptr;
            TRY(launch_proj(c, m, a, EPI_RESID, tiled ? m.t_wo[l] : nullptr, d, &slots, nullptr, 5));
        }
        {   // gate / up projections + SwiGLU
            GemvArgs a = base(d, m.xg, m.xgb, xgb_lo);
            a.w0 = m.wg[l]; a.w1 = m.wu[l]; a.n0 = ffn;
            a.ssq_in = m.ssq; a.ssq_in_slots = slots;
            a.y = m.act; a.yb = m.actb; a.yb_lo = actb_lo;
            a.wscale = tiled ? m.sc_gu[l] : nullptr;
            TRY(launch_proj(c, m, a, EPI_SWIGLU, tiled ? m.t_gu[l] : nullptr, 2 * ffn, nullptr, nullptr));
        }
        {   // down projection + residual
            GemvArgs a = base(ffn, m.act, m.actb, actb_lo);
            a.w0 = m.wd[l]; a.n0 = d;
            a.xres = m.x; a.g_next = (l + 1 < s.n_layers) ? m.attn_norm[l + 1] : m.final_norm;
            a.xg = m.xg; a.xgb = m.xgb; a.xgb_lo = xgb_lo; a.ssq_out = m.ssq;
            a.wscale = tiled ? m.sc_wd[l] : nullptr;
            TRY(launch_proj(c, m, a, EPI_RESID, tiled ? m.t_wd[l] : nullptr, d, &slots, nullptr, 6));
        }
    }
    if (lp.want) {
        GemvArgs a = base(d, m.xg, m.xgb, xgb_lo);
        a.R = lp.rows;
        a.x_mul = lp.x_mul; a.x_add = lp.x_add;
        a.w0 = m.lm_head; a.n0 = s.vocab;
        a.ssq_in = m.ssq; a.ssq_in_slots = slots;
        a.y = m.logits; a.y_mul = lp.y_mul; a.y_add = lp.y_add; a.y_rows = lp.y_rows; a.y_stride = s.vocab;
        a.pm = m.pm; a.ps = m.ps; a.pa = m.pa; a.inv_t = c->scfg.inv_t;
        int nb = 0, tile = 0;
        a.wscale = tiled ? m.sc_lm : nullptr;
        TRY(launch_proj(c, m, a, EPI_LOGITS, tiled ? m.t_lm : nullptr, s.vocab, &nb, &tile));
        *lp.tile = tile;
        *lp.ntiles = nb;
        HIPCHK(c, launch_merge_partials(m.pm, m.ps, m.pa, nb, c->scfg.inv_t, m.pm2, m.ps2, m.pa2, lp.rows, lp.y_mul, lp.y_add,
                                        lp.y_rows, active, st));
    }
    return SPEC_OK;
}

// One draft pass: forward of the draft model and the sampler; pass 1 also opens the step.
// `rows` > 0 (passes after the first): only the `rows` sequences that still draft have a row, in sequence order
// (embed_k finds them from the device's own k[b]); the caller knows their number from the planned gammas or from
// what the previous pass's sampler reported.  The sampler works per sequence either way.
int enqueue_draft_pass(spec_ctx *c, int j, int rows = 0) {
    if (j == 1) HIPCHK(c, launch_begin_draft(c->st, c->d_gamma_plan, c->stream));
    const int B = c->cfg.batch;
    RowPlan plan{};
    LogitsPlan lp{};
    lp.want = true;
    lp.rows = rows > 0 ? rows : B;
    lp.tile = &c->d_tile;
    lp.ntiles = &c->d_ntiles;
    lp.y_mul = c->cfg.gamma_max;
    lp.y_add = j - 1;
    if (j == 1) {
        plan.mode = ROWS_DRAFT_FIRST; plan.rps = 2; plan.arg = 0;
        lp.x_mul = 2; lp.x_add = 1;
    } else {
        plan.mode = ROWS_DRAFT_NEXT; plan.rps = 1; plan.arg = j;
        lp.x_mul = 1; lp.x_add = 0;
        if (rows > 0) { plan.ragged = 1; lp.y_rows = c->drf.row_seq; }
    }
    TRY(forward(c, c->drf, plan, lp, true, rows));
    DraftSampleArgs a{};
    a.st = c->st; a.cfg = c->scfg; a.j = j; a.gamma_max = c->cfg.gamma_max; a.logits = c->drf.logits;
    a.vocab = c->drf.s.vocab; a.pm = c->drf.pm; a.ps = c->drf.ps; a.pa = c->drf.pa;
    a.n_tiles = c->d_ntiles; a.tile = c->d_tile;
    a.pm2 = c->drf.pm2; a.ps2 = c->drf.ps2; a.pa2 = c->drf.pa2; a.n2 = (c->d_ntiles + 63) / 64;
    a.host_pass = c->d_pass;
    a.q_logit = c->q_logit; a.q_max = c->q_max; a.q_sum = c->q_sum;
    HIPCHK(c, launch_draft_sample(a, c->stream));
    return SPEC_OK;
}

int enqueue_draft(spec_ctx *c, int gamma) {
    for (int j = 1; j <= gamma; ++j) TRY(enqueue_draft_pass(c, j));
    return SPEC_OK;
}

// Wait until the device has sampled `n` draft passes since the last reset; *active = sequences still drafting.
int wait_draft_pass(spec_ctx *c, int n, int *active) {
    const auto t0 = std::chrono::steady_clock::now();
    for (uint64_t spins = 0;; ++spins) {
        if (__atomic_load_n(&c->h_pass[0], __ATOMIC_ACQUIRE) >= n) break;
        if ((spins & 0xffff) == 0xffff &&
            std::chrono::steady_clock::now() - t0 > std::chrono::seconds(20)) {
            const hipError_t e = hipStreamQuery(c->stream);
            return fail(c, SPEC_EHIP, std::string("draft pass did not report within 20 s: ") + hipGetErrorString(e));
        }
    }
    *active = __atomic_load_n(&c->h_pass[1], __ATOMIC_RELAXED);
    return SPEC_OK;
}

// `rows_total` > 0: the sequences differ in their planned gamma and the pass holds only the gamma_b + 1 rows each
// of them planned, one sequence after the other.
int enqueue_verify(spec_ctx *c, int gamma, int rows_total) {
    RowPlan plan{};
    plan.mode = ROWS_VERIFY; plan.rps = gamma + 1; plan.arg = 0; plan.ragged = rows_total > 0;
    LogitsPlan lp{};
    lp.want = true;
    lp.rows = rows_total > 0 ? rows_total : c->cfg.batch * (gamma + 1);
    lp.tile = &c->t_tile;
    lp.ntiles = &c->t_ntiles;
    return forward(c, c->tgt, plan, lp, false, rows_total);
}

int enqueue_accept(spec_ctx *c, int gamma) {
    AcceptArgs a{};
    a.st = c->st; a.cfg = c->scfg; a.gamma = gamma; a.gamma_max = c->cfg.gamma_max; a.vocab = c->tgt.s.vocab;
    a.p_logits = c->tgt.logits; a.row_off = c->cur_rows > 0 ? c->tgt.row_off : nullptr; a.pm = c->tgt.pm; a.ps = c->tgt.ps; a.pa = c->tgt.pa;
    a.n_tiles = c->t_ntiles; a.tile = c->t_tile;
    a.pm2 = c->tgt.pm2; a.ps2 = c->tgt.ps2; a.pa2 = c->tgt.pa2; a.n2 = (c->t_ntiles + 63) / 64;
    a.q_logits = c->drf.logits; a.q_logit = c->q_logit; a.q_max = c->q_max; a.q_sum = c->q_sum;
    a.row_max = c->row_max; a.row_sum = c->row_sum; a.row_arg = c->row_arg; a.resid_row = c->resid_row;
    a.resid_part = c->resid_part; a.n_resid_chunks = RESID_CHUNKS; a.ticket = c->ticket;
    a.out_A = c->d_out; a.out_y = c->d_out + c->cfg.batch; a.out_k = c->d_out + 2 * c->cfg.batch;
    a.A_dev = c->A_dev; a.y_dev = c->y_dev;
    HIPCHK(c, launch_accept(a, c->stream));
    return SPEC_OK;
}

// Capture `body` into an executable graph.
template <typename F> int capture(spec_ctx *c, F body, hipGraphExec_t *out) {
    HIPCHK(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
    c->capturing = true;
    const int rc = body();
    c->capturing = false;
    hipGraph_t g = nullptr;
    const hipError_t e = hipStreamEndCapture(c->stream, &g);
    if (rc != SPEC_OK) {
        if (g) (void)hipGraphDestroy(g);
        return rc;
    }
    if (e != hipSuccess) return fail(c, SPEC_EHIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
    c->graphs.push_back(g);
    HIPCHK(c, hipGraphInstantiate(out, g, nullptr, nullptr, 0));
    return SPEC_OK;
}

int prefill_model(spec_ctx *c, ModelRT &m, int n_ingest) {
    const int B = c->cfg.batch;
    const int chunk = std::max(1, ingest_rows(c->cfg, m.s) / B);
    for (int p0 = 0; p0 < n_ingest; p0 += chunk) {
        RowPlan plan{};
        plan.mode = ROWS_PREFILL;
        plan.rps = std::min(chunk, n_ingest - p0);
        plan.arg = p0;
        LogitsPlan lp{};
        TRY(forward(c, m, plan, lp, false));
    }
    return SPEC_OK;
}


// ---- stand-alone accept / resample: scratch layout, kernels and launch sequence shared by its two entry points ----
struct AcceptScratch {
    size_t o_ps, o_qs, o_rmax, o_rsum, o_part, o_qsum, o_pm, o_qm, o_pa, o_qa, o_ql, o_qmax, o_rarg, o_tok, o_state,
        o_ps2, o_pm2, o_pa2, total;
    int n_tiles, n2;
};
constexpr int ACCEPT_TILE = 256;

constexpr size_t accept_scratch_bytes(int k, int vocab) {
    // mirrors accept_scratch_layout(): every block rounded up to 256 bytes
    const size_t rp = (size_t)k + 1, rq = (size_t)k, nt = (size_t)((vocab + ACCEPT_TILE - 1) / ACCEPT_TILE), n2 = (nt + 63) / 64;
    size_t off = 0;
    const size_t blocks[] = {rp * nt * 8, rq * nt * 8, rp * 8, rp * 8, (size_t)RESID_CHUNKS * 8, rq * 8, rp * nt * 4, rq * nt * 4,
                             rp * nt * 4, rq * nt * 4, rq * 4, rq * 4, rp * 4, (rp + 1) * 4, 64 * 4, rp * n2 * 8, rp * n2 * 4,
                             rp * n2 * 4};
    for (size_t b : blocks) off += (b + 255) & ~(size_t)255;
    return off;
}

AcceptScratch accept_scratch_layout(int k, int vocab) {
    AcceptScratch L{};
    L.n_tiles = (vocab + ACCEPT_TILE - 1) / ACCEPT_TILE;
    L.n2 = (L.n_tiles + 63) / 64;
    const size_t rows_p = (size_t)k + 1, rows_q = (size_t)k, nt = (size_t)L.n_tiles, n2 = (size_t)L.n2;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
    L.o_ps = take(rows_p * nt * 8); L.o_qs = take(rows_q * nt * 8); L.o_rmax = take(rows_p * 8); L.o_rsum = take(rows_p * 8);
    L.o_part = take((size_t)RESID_CHUNKS * 8); L.o_qsum = take(rows_q * 8); L.o_pm = take(rows_p * nt * 4);
    L.o_qm = take(rows_q * nt * 4); L.o_pa = take(rows_p * nt * 4); L.o_qa = take(rows_q * nt * 4); L.o_ql = take(rows_q * 4);
    L.o_qmax = take(rows_q * 4); L.o_rarg = take(rows_p * 4); L.o_tok = take((rows_p + 1) * 4); L.o_state = take(64 * 4);
    L.o_ps2 = take(rows_p * n2 * 8); L.o_pm2 = take(rows_p * n2 * 4); L.o_pa2 = take(rows_p * n2 * 4);
    L.total = off;
    return L;
}

// Row partials, their merge, the draft-side statistics and the accept kernels on a zeroed scratch block whose
// state words and drafted tokens are already in place.  state ints: [0] len = 0, [1] prompt_len = 0, [2] gamma_b,
// [3] k, [4..7] ctl, [8] resid_row, [9] ticket, [10] A, [11] y, [12] out_A, [13] out_y, [14] out_k.
hipError_t accept_on_scratch(uint8_t *buf, const AcceptScratch &L, const float *p_logits, const float *q_logits,
                             const int32_t *drafted, int k, int vocab, float temperature, uint64_t seed, hipStream_t st) {
    const float inv_t = temperature > 0.f ? 1.f / temperature : 1.f;
    const int n_tiles = L.n_tiles, n2 = L.n2, tile = ACCEPT_TILE;
    hipError_t e;
    int32_t *state = reinterpret_cast<int32_t *>(buf + L.o_state);
    int32_t *tok = reinterpret_cast<int32_t *>(buf + L.o_tok);
    float *pm = reinterpret_cast<float *>(buf + L.o_pm), *qm = reinterpret_cast<float *>(buf + L.o_qm);
    double *ps = reinterpret_cast<double *>(buf + L.o_ps), *qs = reinterpret_cast<double *>(buf + L.o_qs);
    int32_t *pa = reinterpret_cast<int32_t *>(buf + L.o_pa), *qa = reinterpret_cast<int32_t *>(buf + L.o_qa);
    if ((e = launch_row_partials(p_logits, k + 1, vocab, tile, inv_t, pm, ps, pa, st)) != hipSuccess) return e;
    if ((e = launch_row_partials(q_logits, k, vocab, tile, inv_t, qm, qs, qa, st)) != hipSuccess) return e;
    float *pm2 = reinterpret_cast<float *>(buf + L.o_pm2);
    double *ps2 = reinterpret_cast<double *>(buf + L.o_ps2);
    int32_t *pa2 = reinterpret_cast<int32_t *>(buf + L.o_pa2);
    if ((e = launch_merge_partials(pm, ps, pa, n_tiles, inv_t, pm2, ps2, pa2, k + 1, 1, 0, nullptr, nullptr, st)) != hipSuccess) return e;
    float *ql = reinterpret_cast<float *>(buf + L.o_ql), *qmax = reinterpret_cast<float *>(buf + L.o_qmax);
    double *qsum = reinterpret_cast<double *>(buf + L.o_qsum);
    if ((e = launch_gather_qstats(q_logits, drafted, k, vocab, qm, qs, qa, n_tiles, inv_t, ql, qmax, qsum, st)) != hipSuccess) return e;
    AcceptArgs a{};
    a.st.len = state; a.st.prompt_len = state + 1; a.st.gamma_b = state + 2; a.st.k = state + 3; a.st.ctl = state + 4;
    a.st.tokens = tok; a.st.max_seq = k + 2; a.st.batch = 1;
    a.cfg.temperature = temperature; a.cfg.inv_t = inv_t; a.cfg.seed = seed; a.cfg.forced = 0; a.cfg.tau = 0.f;
    a.cfg.alpha = nullptr; a.cfg.n_alpha = 0;
    a.gamma = k; a.gamma_max = k; a.vocab = vocab; a.p_logits = p_logits; a.pm = pm; a.ps = ps; a.pa = pa;
    a.n_tiles = n_tiles; a.tile = tile; a.pm2 = pm2; a.ps2 = ps2; a.pa2 = pa2; a.n2 = n2; a.q_logits = q_logits; a.q_logit = ql; a.q_max = qmax; a.q_sum = qsum;
    a.row_max = reinterpret_cast<double *>(buf + L.o_rmax); a.row_sum = reinterpret_cast<double *>(buf + L.o_rsum);
    a.row_arg = reinterpret_cast<int32_t *>(buf + L.o_rarg); a.resid_row = state + 8;
    a.resid_part = reinterpret_cast<double *>(buf + L.o_part); a.n_resid_chunks = RESID_CHUNKS;
    a.ticket = reinterpret_cast<uint32_t *>(state + 9);
    a.A_dev = state + 10; a.y_dev = state + 11; a.out_A = state + 12; a.out_y = state + 13; a.out_k = state + 14;
    return launch_accept(a, st);
}

// Scratch of spec_k_accept_static: one array per GPU the library runs on, held until the process ends; sized for
// the largest call the entry point admits.  Host code never uses the array's name as an address: the device
// address is looked up once per device (accept_static_scratch) and passed to the kernels like any other buffer.
constexpr int SPEC_ACCEPT_STATIC_MAX_K = 64;
constexpr int SPEC_ACCEPT_STATIC_MAX_VOCAB = 262144;
constexpr size_t ACCEPT_STATIC_BYTES = accept_scratch_bytes(SPEC_ACCEPT_STATIC_MAX_K, SPEC_ACCEPT_STATIC_MAX_VOCAB);
static __device__ __align__(256) unsigned char g_accept_scratch[ACCEPT_STATIC_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
uint8_t *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of the current device's copy of the array (looked up on the first call per device).
int accept_static_scratch(uint8_t **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return fail(nullptr, SPEC_EHIP, "accept_static: no current device");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_accept_scratch));
        if (e != hipSuccess || p == nullptr)
            return fail(nullptr, SPEC_EHIP, std::string("accept_static: hipGetSymbolAddress: ") + hipGetErrorString(e));
        g_scratch_ptr[dev] = reinterpret_cast<uint8_t *>(p);
    }
    *out = g_scratch_ptr[dev];
    return SPEC_OK;
}

// Start state of one stand-alone accept call in its scratch block: the first n16 16-byte words are zeroed, except
// the state words (gamma_b = k, drafted count = k, step ordinal) and the token slots (the drafted tokens), which the
// threads that would otherwise zero them write instead, so that no word has two writers.  A kernel rather than a
// memset and copies: the caller may be capturing the stream.
__global__ __launch_bounds__(256) void accept_scratch_init_k(uint4 *buf, int n16, int32_t *state, int32_t *tok,
                                                             const int32_t *drafted, int k, int step) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    const uint4 *s16 = reinterpret_cast<const uint4 *>(state), *t16 = reinterpret_cast<const uint4 *>(tok);
    const int s_first = (int)(s16 - buf), t_first = (int)(t16 - buf);
    if (i >= n16) return;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (i >= s_first && i < s_first + 4) {
        int32_t w[4] = {0, 0, 0, 0};
        for (int j = 0; j < 4; ++j) {
            const int idx = (i - s_first) * 4 + j;
            w[j] = idx == 2 || idx == 3 ? k : (idx == 4 ? step : 0);
        }
        v = make_uint4((uint32_t)w[0], (uint32_t)w[1], (uint32_t)w[2], (uint32_t)w[3]);
    } else if (i >= t_first && i < t_first + (k + 3) / 4) {
        int32_t w[4];
        for (int j = 0; j < 4; ++j) {
            const int idx = (i - t_first) * 4 + j;
            w[j] = idx < k ? drafted[idx] : 0;
        }
        v = make_uint4((uint32_t)w[0], (uint32_t)w[1], (uint32_t)w[2], (uint32_t)w[3]);
    }
    buf[i] = v;
}

__global__ void accept_result_k(const int32_t *out, int32_t *result) {
    if (threadIdx.x < 2) result[threadIdx.x] = out[threadIdx.x];
}

}  // namespace

extern "C" {

const char *spec_strerror(int code) {
    switch (code) {
        case SPEC_OK: return "ok";
        case SPEC_EINVAL: return "invalid argument";
        case SPEC_ESTATE: return "call order violated";
        case SPEC_ENOMEM: return "out of memory";
        case SPEC_EHIP: return "HIP runtime error";
        case SPEC_ECAP: return "sequence capacity exceeded";
        case SPEC_ENOTIMPL: return "not implemented";
    }
    return "unknown error";
}

const char *spec_last_error(const spec_ctx *ctx) { return ctx ? ctx->err.c_str() : g_last_err.c_str(); }

int64_t spec_device_bytes(const spec_ctx *ctx) { return ctx ? ctx->dev_bytes : 0; }

void spec_destroy(spec_ctx *c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    for (auto &kv : c->g_draft) (void)hipGraphExecDestroy(kv.second);
    for (auto &kv : c->g_verify) (void)hipGraphExecDestroy(kv.second.exec);
    for (auto &kv : c->g_pass) (void)hipGraphExecDestroy(kv.second);
    for (auto g : c->graphs) (void)hipGraphDestroy(g);
    for (void *p : c->dev_allocs) (void)hipFree(p);
    for (void *p : c->host_allocs) (void)hipHostFree(p);
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
    if (c->own_stream) (void)hipStreamDestroy(c->stream);
    delete c;
}

int spec_init(const spec_shape *t, const spec_weights *tw, const spec_shape *d, const spec_weights *dw,
              const spec_config *cfg, spec_ctx **out) {
    if (!out) return SPEC_EINVAL;
    *out = nullptr;
    if (!t || !tw || !d || !dw || !cfg) return SPEC_EINVAL;
    spec_ctx *c = new spec_ctx();
    auto bail = [&](int rc) {  // the message stays reachable through spec_last_error(NULL)
        spec_destroy(c);
        return rc;
    };
    c->cfg = *cfg;
    if (c->cfg.page_tokens == 0) c->cfg.page_tokens = 64;
    c->stream = reinterpret_cast<hipStream_t>(cfg->hip_stream);
    // whatever produced the weights (on any stream) must have finished before they are read here
    if (hipDeviceSynchronize() != hipSuccess) return bail(fail(c, SPEC_EHIP, "init: device sync failed"));
    if (c->stream == nullptr) {
        // the null stream cannot be captured into a graph: work runs on a stream of the context's own
        if (hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking) != hipSuccess)
            return bail(fail(c, SPEC_EHIP, "init: hipStreamCreate failed"));
        c->own_stream = true;
    }
    int rc;
    {   // the fixed scratch array of spec_k_accept_static: its address on this device is looked up at set-up, so that
        // a first call made under stream capture finds it ready
        uint8_t *scratch = nullptr;
        if ((rc = accept_static_scratch(&scratch))) return bail(rc);
    }
    if ((rc = check_shape(c, *t, "target")) || (rc = check_shape(c, *d, "draft")) ||
        (rc = check_weights(c, *t, tw, "target")) || (rc = check_weights(c, *d, dw, "draft")))
        return bail(rc);
    const spec_config &g = c->cfg;
    if (t->vocab != d->vocab) return bail(fail(c, SPEC_EINVAL, "draft and target vocabularies differ"));
    if (g.batch < 1 || g.batch > 64) return bail(fail(c, SPEC_EINVAL, "batch outside 1..64"));
    if (g.gamma_max < 1 || g.gamma_max > 64) return bail(fail(c, SPEC_EINVAL, "gamma_max outside 1..64"));
    if (g.page_tokens < 8 || (g.page_tokens & (g.page_tokens - 1)))
        return bail(fail(c, SPEC_EINVAL, "page_tokens must be a power of two >= 8"));
    if (g.attn_chunk != 0 && g.attn_chunk != 64 && g.attn_chunk != 128 && g.attn_chunk != 256 && g.attn_chunk != 512)
        return bail(fail(c, SPEC_EINVAL, "attn_chunk must be 0, 64, 128, 256 or 512"));
    if (g.max_seq < g.gamma_max + 2) return bail(fail(c, SPEC_EINVAL, "max_seq too small"));
    if (!(g.temperature >= 0.f)) return bail(fail(c, SPEC_EINVAL, "temperature < 0"));
    if (g.accept_mode != SPEC_ACCEPT_NATURAL && g.accept_mode != SPEC_ACCEPT_FORCED)
        return bail(fail(c, SPEC_EINVAL, "unknown accept_mode"));
    {   // rows of a verification pass: 128 on the weight-streaming kernels; up to the ingestion launch size when
        // the target also runs on the dense-contraction kernels.  The first draft pass has two rows per sequence.
        const int rows = g.batch * (g.gamma_max + 1);
        const int cap = ingest_rows(c->cfg, *t) >= PREFILL_GEMM_ROWS ? PREFILL_GEMM_ROWS : 128;
        if (rows > cap) return bail(fail(c, SPEC_EINVAL, "batch * (gamma_max + 1) exceeds the rows of one pass (128, or 1024 for a bf16 target on the matrix cores)"));
        if (2 * g.batch > 128) return bail(fail(c, SPEC_EINVAL, "batch > 64"));
    }

    const int B = g.batch;
    const int rows_t = std::max(B * (g.gamma_max + 1), ingest_rows(c->cfg, *t));
    const int rows_d = std::max(2 * B, ingest_rows(c->cfg, *d));
    if ((rc = build_model(c, c->tgt, *t, tw, rows_t, B * (g.gamma_max + 1)))) return bail(rc);
    if ((rc = build_model(c, c->drf, *d, dw, rows_d, B * g.gamma_max))) return bail(rc);

    auto A = [&](auto **p, size_t n) { return dalloc(c, p, n); };
    if ((rc = A(&c->st.len, B)) || (rc = A(&c->st.prompt_len, B)) || (rc = A(&c->st.gamma_b, B)) ||
        (rc = A(&c->st.k, B)) || (rc = A(&c->st.ctl, 4)) || (rc = A(&c->st.tokens, (size_t)B * g.max_seq)) ||
        (rc = A(&c->q_logit, (size_t)B * g.gamma_max)) || (rc = A(&c->q_max, (size_t)B * g.gamma_max)) ||
        (rc = A(&c->q_sum, (size_t)B * g.gamma_max)) || (rc = A(&c->row_max, (size_t)B * (g.gamma_max + 1))) ||
        (rc = A(&c->row_sum, (size_t)B * (g.gamma_max + 1))) || (rc = A(&c->row_arg, (size_t)B * (g.gamma_max + 1))) ||
        (rc = A(&c->resid_row, B)) || (rc = A(&c->resid_part, (size_t)B * RESID_CHUNKS)) || (rc = A(&c->ticket, B)) ||
        (rc = A(&c->A_dev, B)) || (rc = A(&c->y_dev, B)) || (rc = A(&c->d_alpha, 1)))
        return bail(rc);
    c->st.max_seq = g.max_seq;
    c->st.batch = B;
    c->ragged_ok = B > 1 && model_on_matrix_cores(c->cfg, *t) && attention_on_matrix_cores(c->cfg, *t);
    c->compact_ok = B > 1 && model_on_matrix_cores(c->cfg, *d) && attention_on_matrix_cores(c->cfg, *d) &&
                    std::getenv("SPEC_NO_DRAFT_COMPACT") == nullptr;
    c->h_len.assign(B, 0);

    void *hp = nullptr;
    if (hipHostMalloc(&hp, sizeof(int32_t) * (4 * B + 2), hipHostMallocMapped) != hipSuccess)
        return bail(fail(c, SPEC_ENOMEM, "hipHostMalloc failed"));
    c->host_allocs.push_back(hp);
    std::memset(hp, 0, sizeof(int32_t) * (4 * B + 2));
    c->h_gamma_plan = reinterpret_cast<int32_t *>(hp);
    c->h_out = c->h_gamma_plan + B;
    c->h_pass = c->h_gamma_plan + 4 * B;
    void *dp = nullptr;
    if (hipHostGetDevicePointer(&dp, hp, 0) != hipSuccess)
        return bail(fail(c, SPEC_EHIP, "hipHostGetDevicePointer failed"));
    c->d_gamma_plan = reinterpret_cast<int32_t *>(dp);
    c->d_out = c->d_gamma_plan + B;
    c->d_pass = c->d_gamma_plan + 4 * B;

    c->scfg.temperature = g.temperature;
    c->scfg.inv_t = g.temperature > 0.f ? 1.0f / g.temperature : 1.0f;
    c->scfg.seed = g.seed;
    c->scfg.forced = g.accept_mode == SPEC_ACCEPT_FORCED;
    c->scfg.alpha = c->d_alpha;
    c->scfg.n_alpha = 1;
    c->scfg.tau = 0.f;
    {
        const float one = 1.0f;
        if (hipStreamSynchronize(c->stream) != hipSuccess) return bail(fail(c, SPEC_EHIP, "init: stream sync failed"));
        if (hipMemcpy(c->d_alpha, &one, sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
            return bail(fail(c, SPEC_EHIP, "hipMemcpy failed"));
    }
    if (hipStreamSynchronize(c->stream) != hipSuccess) return bail(fail(c, SPEC_EHIP, "init: stream sync failed"));
    *out = c;
    return SPEC_OK;
}

int spec_set_forced_alpha(spec_ctx *c, const float *alpha, int32_t n) {
    if (!c || !alpha || n < 1) return fail(c, SPEC_EINVAL, "set_forced_alpha: bad arguments");
    for (int i = 0; i < n; ++i)
        if (!(alpha[i] >= 0.f && alpha[i] <= 1.f)) return fail(c, SPEC_EINVAL, "alpha outside [0,1]");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    float *p = nullptr;
    TRY(dalloc(c, &p, (size_t)n));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(p, alpha, sizeof(float) * n, hipMemcpyHostToDevice));
    c->d_alpha = p;
    c->scfg.alpha = p;
    c->scfg.n_alpha = n;
    // kernel arguments are baked into captured graphs
    for (auto &kv : c->g_draft) (void)hipGraphExecDestroy(kv.second);
    for (auto &kv : c->g_verify) (void)hipGraphExecDestroy(kv.second.exec);
    for (auto &kv : c->g_pass) (void)hipGraphExecDestroy(kv.second);
    c->g_draft.clear();
    c->g_verify.clear();
    c->g_pass.clear();
    return SPEC_OK;
}

int spec_set_early_stop(spec_ctx *c, float tau) {
    if (!c) return SPEC_EINVAL;
    if (!(tau == tau)) return fail(c, SPEC_EINVAL, "tau is NaN");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->scfg.tau = tau > 0.f ? tau : 0.f;
    for (auto &kv : c->g_draft) (void)hipGraphExecDestroy(kv.second);
    c->g_draft.clear();
    for (auto &kv : c->g_pass) (void)hipGraphExecDestroy(kv.second);
    c->g_pass.clear();
    return SPEC_OK;
}

int spec_debug_set_block_table(spec_ctx *c, const int32_t *table) {
    if (!c || !table) return SPEC_EINVAL;
    if (c->prefilled) return fail(c, SPEC_ESTATE, "block table must be set before prefill");
    for (ModelRT *m : {&c->tgt, &c->drf}) {
        std::vector<char> seen((size_t)m->n_pages, 0);
        for (int i = 0; i < m->n_pages; ++i) {
            if (table[i] < 0 || table[i] >= m->n_pages || seen[(size_t)table[i]])
                return fail(c, SPEC_EINVAL, "block table is not a permutation");
            seen[(size_t)table[i]] = 1;
        }
        HIPCHK(c, hipMemcpy(m->block_table, table, sizeof(int32_t) * m->n_pages, hipMemcpyHostToDevice));
    }
    return SPEC_OK;
}

int spec_prefill_ragged(spec_ctx *c, const int32_t *host_tokens, int32_t n_max, const int32_t *lens) {
    if (!c || !host_tokens || !lens) return fail(c, SPEC_EINVAL, "prefill: null pointer");
    const int B = c->cfg.batch;
    if (n_max < 1 || n_max + c->cfg.gamma_max + 1 > c->cfg.max_seq) return fail(c, SPEC_ECAP, "prefill: prompt does not fit max_seq");
    for (int b = 0; b < B; ++b) {
        if (lens[b] < 1 || lens[b] > n_max) return fail(c, SPEC_EINVAL, "prefill: length outside 1..n_max");
        for (int i = 0; i < lens[b]; ++i) {
            const int32_t t = host_tokens[(size_t)b * n_max + i];
            if (t < 0 || t >= c->tgt.s.vocab) return fail(c, SPEC_EINVAL, "prefill: token id out of range");
        }
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    std::vector<int32_t> toks((size_t)B * c->cfg.max_seq, 0);
    for (int b = 0; b < B; ++b)
        std::memcpy(&toks[(size_t)b * c->cfg.max_seq], host_tokens + (size_t)b * n_max, sizeof(int32_t) * lens[b]);
    HIPCHK(c, hipMemcpy(c->st.tokens, toks.data(), toks.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(c->st.len, lens, sizeof(int32_t) * B, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(c->st.prompt_len, lens, sizeof(int32_t) * B, hipMemcpyHostToDevice));
    const int32_t ctl[4] = {-1, 0, 0, 0};
    HIPCHK(c, hipMemcpy(c->st.ctl, ctl, sizeof(ctl), hipMemcpyHostToDevice));
    c->passes_launched = 0;
    c->h_pass[0] = 0;
    c->h_pass[1] = 0;
    std::vector<uint32_t> z(B, 0);
    HIPCHK(c, hipMemcpy(c->ticket, z.data(), sizeof(uint32_t) * B, hipMemcpyHostToDevice));
    c->h_len.assign(lens, lens + B);
    // every sequence ingests positions 0 .. n_max-2; rows past a shorter sequence's end hold padding
    // tokens whose cache entries are rewritten by the decode steps before anything reads them
    // the two models share nothing they write: the draft ingests on a stream of its own beside the target (both are
    // bound by load latency rather than by throughput, so their kernels interleave to a shorter whole)
    // (SPEC_PREFILL_ONE_STREAM in the environment keeps both on the context's stream: kernel traces whose durations
    // do not overlap)
    static const bool one_stream = std::getenv("SPEC_PREFILL_ONE_STREAM") != nullptr;
    if (!one_stream && c->side_stream == nullptr) HIPCHK(c, hipStreamCreateWithFlags(&c->side_stream, hipStreamNonBlocking));
    TRY(prefill_model(c, c->tgt, n_max - 1));
    if (one_stream) {
        TRY(prefill_model(c, c->drf, n_max - 1));
    } else {
        const hipStream_t main_stream = c->stream;
        c->stream = c->side_stream;
        const int rc_d = prefill_model(c, c->drf, n_max - 1);
        c->stream = main_stream;
        const hipError_t e_d = hipStreamSynchronize(c->side_stream);
        if (rc_d != SPEC_OK) return rc_d;
        HIPCHK(c, e_d);
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->prefilled = true;
    c->phase = 1;
    return SPEC_OK;
}

int spec_prefill(spec_ctx *c, const int32_t *host_tokens, int32_t n) {
    if (!c) return SPEC_EINVAL;
    std::vector<int32_t> lens((size_t)c->cfg.batch, n);
    return spec_prefill_ragged(c, host_tokens, n, lens.data());
}

int spec_debug_set_step(spec_ctx *c, int32_t step, const int32_t *prompt_lens) {
    if (!c || !prompt_lens) return fail(c, SPEC_EINVAL, "set_step: null pointer");
    if (c->phase != 1) return fail(c, SPEC_ESTATE, "set_step: expected after prefill or accept");
    if (step < 0) return fail(c, SPEC_EINVAL, "set_step: negative step");
    for (int b = 0; b < c->cfg.batch; ++b)
        if (prompt_lens[b] < 1 || prompt_lens[b] > c->h_len[b]) return fail(c, SPEC_EINVAL, "set_step: bad prompt length");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const int32_t before = step - 1;  // the draft phase increments the ordinal first
    HIPCHK(c, hipMemcpy(c->st.ctl, &before, sizeof(int32_t), hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(c->st.prompt_len, prompt_lens, sizeof(int32_t) * c->cfg.batch, hipMemcpyHostToDevice));
    return SPEC_OK;
}

int spec_draft_batch(spec_ctx *c, const int32_t *gammas) {
    if (!c || !gammas) return fail(c, SPEC_EINVAL, "draft: null pointer");
    if (c->phase != 1) return fail(c, SPEC_ESTATE, "draft: expected after prefill or accept");
    const int B = c->cfg.batch;
    int gmax = 0;
    for (int b = 0; b < B; ++b) {
        if (gammas[b] < 1 || gammas[b] > c->cfg.gamma_max) return fail(c, SPEC_EINVAL, "draft: gamma outside 1..gamma_max");
        gmax = std::max(gmax, gammas[b]);
    }
    for (int b = 0; b < B; ++b)
        if (c->h_len[b] + gmax + 1 > c->cfg.max_seq) return fail(c, SPEC_ECAP, "draft: len + gamma + 1 > max_seq");
    for (int b = 0; b < B; ++b) c->h_gamma_plan[b] = gammas[b];
    // One pass, with a row for every sequence (rows == 0) or only for the `rows` sequences that still draft.
    auto launch_pass = [&](int j, int rows) -> int {
        if (rows >= B) rows = 0;
        if (c->cfg.use_graphs) {
            const int key = rows * 128 + j;  // j <= 64
            auto it = c->g_pass.find(key);
            if (it == c->g_pass.end()) {
                hipGraphExec_t ex = nullptr;
                TRY(capture(c, [&] { return enqueue_draft_pass(c, j, rows); }, &ex));
                it = c->g_pass.emplace(key, ex).first;
            }
            HIPCHK(c, hipGraphLaunch(it->second, c->stream));
        } else {
            TRY(enqueue_draft_pass(c, j, rows));
        }
        c->passes_launched += 1;
        return SPEC_OK;
    };
    bool differ = false;
    for (int b = 1; b < B; ++b) differ = differ || gammas[b] != gammas[0];
    if (c->scfg.tau > 0.f && gmax > 1) {
        // early stopping: pass by pass, and the next pass only while a sequence still drafts - over those sequences
        // alone where the draft model's kernels take packed rows
        for (int j = 1; j <= gmax; ++j) {
            int active = B;
            if (j > 1) {
                TRY(wait_draft_pass(c, c->passes_launched, &active));
                if (active == 0) break;
            }
            TRY(launch_pass(j, c->compact_ok ? active : 0));
        }
    } else if (c->compact_ok && differ) {
        // planned gammas differ: pass j holds the sequences that planned at least j tokens
        for (int j = 1; j <= gmax; ++j) {
            int rows = 0;
            for (int b = 0; b < B; ++b) rows += gammas[b] >= j;
            TRY(launch_pass(j, rows));
        }
    } else if (c->cfg.use_graphs) {
        auto it = c->g_draft.find(gmax);
        if (it == c->g_draft.end()) {
            hipGraphExec_t ex = nullptr;
            TRY(capture(c, [&] { return enqueue_draft(c, gmax); }, &ex));
            it = c->g_draft.emplace(gmax, ex).first;
        }
        HIPCHK(c, hipGraphLaunch(it->second, c->stream));
        c->passes_launched += gmax;
    } else {
        TRY(enqueue_draft(c, gmax));
        c->passes_launched += gmax;
    }
    c->cur_gamma = gmax;
    c->verify_only_rows = 0;
    c->phase = 2;
    return SPEC_OK;
}

int spec_draft(spec_ctx *c, int32_t gamma) {
    if (!c) return SPEC_EINVAL;
    std::vector<int32_t> g((size_t)c->cfg.batch, gamma);
    return spec_draft_batch(c, g.data());
}

// Enqueue (or replay the graph of) one verification pass of gamma + 1 rows per sequence, or of rows_total packed rows.
static int launch_verify(spec_ctx *c, int gamma, int rows_total) {
    if (c->cfg.use_graphs) {
        const int key = rows_total * 128 + gamma;  // gamma <= 64
        auto it = c->g_verify.find(key);
        if (it == c->g_verify.end()) {
            hipGraphExec_t ex = nullptr;
            TRY(capture(c, [&] { return enqueue_verify(c, gamma, rows_total); }, &ex));
            it = c->g_verify.emplace(key, spec_ctx::VerifyGraph{ex, c->t_tile, c->t_ntiles}).first;
        }
        // the tiling of THIS graph's logits, not of whichever graph was captured last
        c->t_tile = it->second.tile;
        c->t_ntiles = it->second.ntiles;
        HIPCHK(c, hipGraphLaunch(it->second.exec, c->stream));
        return SPEC_OK;
    }
    return enqueue_verify(c, gamma, rows_total);
}

int spec_verify(spec_ctx *c, int32_t gamma) {
    if (!c) return SPEC_EINVAL;
    if (c->phase != 2) return fail(c, SPEC_ESTATE, "verify: expected after draft");
    if (gamma != c->cur_gamma) return fail(c, SPEC_EINVAL, "verify: gamma differs from the draft phase");
    // sequences that planned different gammas: pack only the rows each of them planned
    int rows_total = 0;
    if (c->ragged_ok) {
        int sum = 0;
        for (int b = 0; b < c->cfg.batch; ++b) sum += c->h_gamma_plan[b] + 1;
        if (sum < c->cfg.batch * (gamma + 1)) rows_total = sum;
    }
    c->cur_rows = rows_total;
    TRY(launch_verify(c, gamma, rows_total));
    c->phase = 3;
    return SPEC_OK;
}

int spec_debug_verify_rows(spec_ctx *c, int32_t rows) {
    if (!c) return SPEC_EINVAL;
    if (c->phase != 1) return fail(c, SPEC_ESTATE, "verify_rows: expected after prefill, fill_kv or accept");
    if (rows < 1 || rows > c->cfg.gamma_max + 1) return fail(c, SPEC_EINVAL, "verify_rows: rows outside 1..gamma_max + 1");
    for (int b = 0; b < c->cfg.batch; ++b)
        if (c->h_len[b] - 1 + rows > c->cfg.max_seq) return fail(c, SPEC_ECAP, "verify_rows: rows do not fit max_seq");
    TRY(launch_verify(c, rows - 1, 0));
    c->verify_only_rows = rows;
    c->cur_rows = 0;
    return SPEC_OK;
}

int spec_accept(spec_ctx *c, int32_t *n_accepted, int32_t *next_token, int32_t *n_drafted) {
    if (!c) return SPEC_EINVAL;
    if (c->phase != 3) return fail(c, SPEC_ESTATE, "accept: expected after verify");
    TRY(enqueue_accept(c, c->cur_gamma));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const int B = c->cfg.batch;
    for (int b = 0; b < B; ++b) {
        const int A = c->h_out[b], y = c->h_out[B + b], k = c->h_out[2 * B + b];
        if (n_accepted) n_accepted[b] = A;
        if (next_token) next_token[b] = y;
        if (n_drafted) n_drafted[b] = k;
        c->h_len[b] += A + 1;
    }
    c->phase = 1;
    return SPEC_OK;
}

int spec_generate(spec_ctx *c, gt_state *controllers, int32_t fixed_gamma, int32_t n_generate, spec_gen_stats *stats) {
    if (!c) return SPEC_EINVAL;
    if (n_generate < 0) return fail(c, SPEC_EINVAL, "generate: n_generate < 0");
    if (!controllers && (fixed_gamma < 1 || fixed_gamma > c->cfg.gamma_max))
        return fail(c, SPEC_EINVAL, "generate: fixed gamma outside 1..gamma_max");
    const int B = c->cfg.batch;
    std::vector<int32_t> gam(B), A(B), y(B), k(B), gen(B, 0);
    spec_gen_stats st{};
    for (;;) {
        int least = gen[0];
        for (int b = 1; b < B; ++b) least = std::min(least, gen[b]);
        if (least >= n_generate) break;
        // a sequence that already has its n_generate tokens rides along with the shortest step there is (gamma 1:
        // two rows of the verification pass) until the slowest one is done; its controller is left alone and it
        // stays out of the statistics.  It grows by at most two tokens per step, so 3 * n_generate tokens of
        // room behind the prompt always suffice.
        for (int b = 0; b < B; ++b) gam[b] = gen[b] >= n_generate ? 1 : (controllers ? controllers[b].gamma : fixed_gamma);
        TRY(spec_draft_batch(c, gam.data()));
        TRY(spec_verify(c, c->cur_gamma));
        TRY(spec_accept(c, A.data(), y.data(), k.data()));
        for (int b = 0; b < B; ++b) {
            if (gen[b] >= n_generate) continue;
            if (controllers && gammatune_update(&controllers[b], A[b], k[b]) < 0)
                return fail(c, SPEC_EINVAL, "generate: controller state rejected by gammatune_update");
            gen[b] += A[b] + 1;
            st.accepted += A[b];
            st.drafted += k[b];
            st.gamma_sum += gam[b];
            st.seq_steps += 1;
        }
        st.steps += 1;
    }
    for (int b = 0; b < B; ++b) st.generated += std::min(gen[b], n_generate);
    if (stats) *stats = st;
    return SPEC_OK;
}

int spec_read_tokens(spec_ctx *c, int32_t b, int32_t *host_out, int32_t cap, int32_t *n) {
    if (!c || !host_out || !n) return fail(c, SPEC_EINVAL, "read_tokens: null pointer");
    if (b < 0 || b >= c->cfg.batch) return fail(c, SPEC_EINVAL, "read_tokens: bad sequence index");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const int len = c->h_len[b];
    if (cap < len) return fail(c, SPEC_EINVAL, "read_tokens: buffer too small");
    HIPCHK(c, hipMemcpy(host_out, c->st.tokens + (size_t)b * c->cfg.max_seq, sizeof(int32_t) * len, hipMemcpyDeviceToHost));
    *n = len;
    return SPEC_OK;
}

int spec_debug_logits(spec_ctx *c, int32_t which, float *host_out, int64_t cap, int32_t *rows) {
    if (!c || !host_out || !rows) return fail(c, SPEC_EINVAL, "debug_logits: null pointer");
    if (which != 0 && which != 1) return fail(c, SPEC_EINVAL, "debug_logits: which must be 0 or 1");
    if (which == 1 && c->verify_only_rows > 0) {  // the rows of the last verification-only pass
        HIPCHK(c, hipStreamSynchronize(c->stream));
        const int64_t n = (int64_t)c->cfg.batch * c->verify_only_rows * c->tgt.s.vocab;
        if (cap < n) return fail(c, SPEC_EINVAL, "debug_logits: buffer too small");
        HIPCHK(c, hipMemcpy(host_out, c->tgt.logits, sizeof(float) * (size_t)n, hipMemcpyDeviceToHost));
        *rows = c->verify_only_rows;
        return SPEC_OK;
    }
    if (c->cur_gamma < 1) return fail(c, SPEC_ESTATE, "debug_logits: no step has run");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const int B = c->cfg.batch, V = c->tgt.s.vocab;
    const int rps = which == 0 ? c->cur_gamma : c->cur_gamma + 1;
    if (cap < (int64_t)B * rps * V) return fail(c, SPEC_EINVAL, "debug_logits: buffer too small");
    if (which == 1 && c->cur_rows > 0) {
        // ragged pass: sequence b's gamma_b + 1 rows into its slot of the padded layout, zeros behind them
        std::memset(host_out, 0, sizeof(float) * (size_t)B * rps * V);
        size_t off = 0;
        for (int b = 0; b < B; ++b) {
            const size_t n = (size_t)c->h_gamma_plan[b] + 1;
            HIPCHK(c, hipMemcpy(host_out + (size_t)b * rps * V, c->tgt.logits + off * V, sizeof(float) * n * V, hipMemcpyDeviceToHost));
            off += n;
        }
    } else if (which == 1) {
        HIPCHK(c, hipMemcpy(host_out, c->tgt.logits, sizeof(float) * (size_t)B * rps * V, hipMemcpyDeviceToHost));
    } else {
        for (int b = 0; b < B; ++b)
            HIPCHK(c, hipMemcpy(host_out + (size_t)b * rps * V, c->drf.logits + (size_t)b * c->cfg.gamma_max * V,
                                sizeof(float) * (size_t)rps * V, hipMemcpyDeviceToHost));
    }
    *rows = rps;
    return SPEC_OK;
}

int spec_debug_drafted(spec_ctx *c, int32_t b, int32_t *host_out, int32_t cap, int32_t *n) {
    if (!c || !host_out || !n) return fail(c, SPEC_EINVAL, "debug_drafted: null pointer");
    if (b < 0 || b >= c->cfg.batch) return fail(c, SPEC_EINVAL, "debug_drafted: bad sequence index");
    if (c->phase != 2 && c->phase != 3) return fail(c, SPEC_ESTATE, "debug_drafted: expected between draft and accept");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    int32_t k = 0;
    HIPCHK(c, hipMemcpy(&k, c->st.k + b, sizeof(int32_t), hipMemcpyDeviceToHost));
    if (k < 0 || k > cap) return fail(c, SPEC_EINVAL, "debug_drafted: buffer too small");
    HIPCHK(c, hipMemcpy(host_out, c->st.tokens + (size_t)b * c->cfg.max_seq + c->h_len[b], sizeof(int32_t) * k,
                        hipMemcpyDeviceToHost));
    *n = k;
    return SPEC_OK;
}

int spec_debug_read(spec_ctx *c, int32_t model, int32_t which, void *host_out, int64_t bytes) {
    if (!c || !host_out || bytes < 0) return SPEC_EINVAL;
    ModelRT &m = model ? c->tgt : c->drf;
    const void *src = nullptr;
    switch (which) {
        case 0: src = m.x; break;
        case 1: src = m.q; break;
        case 2: src = m.ao; break;
        case 3: src = m.act; break;
        case 4: src = m.xg; break;
        case 5: src = m.ssq; break;
        case 6: src = m.part_m; break;
        case 7: src = m.part_l; break;
        case 8: src = m.part_o; break;
        case 9: src = m.aob; break;
        case 10: src = m.xgb; break;
        case 11: src = m.actb; break;
        case 12: src = m.qb; break;
        default:
            if (which >= 100 && which < 100 + m.s.n_layers) src = m.kpool[which - 100];
            else if (which >= 200 && which < 200 + m.s.n_layers) src = m.vpool[which - 200];
    }
    if (!src) return fail(c, SPEC_EINVAL, "debug_read: unknown buffer");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(host_out, src, (size_t)bytes, hipMemcpyDeviceToHost));
    return SPEC_OK;
}

int spec_debug_fill_kv(spec_ctx *c, int32_t len, uint64_t seed) {
    if (!c) return SPEC_EINVAL;
    if (len < 0 || len + 1 + c->cfg.gamma_max + 1 > c->cfg.max_seq) return fail(c, SPEC_ECAP, "fill_kv: len does not fit max_seq");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const int B = c->cfg.batch;
    uint64_t sd_ = seed;
    for (ModelRT *m : {&c->tgt, &c->drf}) {
        const int64_t n = (int64_t)m->n_pages * m->s.n_kv_heads * c->cfg.page_tokens * m->s.head_dim;
        for (int l = 0; l < m->s.n_layers; ++l) {
            HIPCHK(c, launch_fill_uniform(m->kpool[l], n, m->s.dtype, sd_++, c->stream));
            HIPCHK(c, launch_fill_uniform(m->vpool[l], n, m->s.dtype, sd_++, c->stream));
        }
    }
    std::vector<int32_t> toks((size_t)B * c->cfg.max_seq, 0);
    HIPCHK(c, hipMemcpy(c->st.tokens, toks.data(), toks.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    std::vector<int32_t> lens(B, len + 1);
    HIPCHK(c, hipMemcpy(c->st.len, lens.data(), sizeof(int32_t) * B, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(c->st.prompt_len, lens.data(), sizeof(int32_t) * B, hipMemcpyHostToDevice));
    const int32_t ctl[4] = {-1, 0, 0, 0};
    HIPCHK(c, hipMemcpy(c->st.ctl, ctl, sizeof(ctl), hipMemcpyHostToDevice));
    c->passes_launched = 0;
    c->h_pass[0] = 0;
    c->h_pass[1] = 0;
    std::vector<uint32_t> z(B, 0);
    HIPCHK(c, hipMemcpy(c->ticket, z.data(), sizeof(uint32_t) * B, hipMemcpyHostToDevice));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->h_len.assign(B, len + 1);
    c->prefilled = true;
    c->phase = 1;
    return SPEC_OK;
}

int spec_debug_write_kv(spec_ctx *c, int32_t model, int32_t layer, int32_t seq, int32_t pos0, int32_t n,
                        const float *k_host, const float *v_host) {
    if (!c || !k_host || !v_host) return SPEC_EINVAL;
    ModelRT &m = model ? c->tgt : c->drf;
    if (layer < 0 || layer >= m.s.n_layers || seq < 0 || seq >= c->cfg.batch || pos0 < 0 || n < 1 ||
        pos0 + n > c->cfg.max_seq)
        return fail(c, SPEC_EINVAL, "write_kv: layer, sequence or positions out of range");
    const size_t count = (size_t)n * m.s.n_kv_heads * m.s.head_dim;
    float *dk = nullptr, *dv = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&dk), count * 4) != hipSuccess) return fail(c, SPEC_ENOMEM, "write_kv: staging");
    if (hipMalloc(reinterpret_cast<void **>(&dv), count * 4) != hipSuccess) { (void)hipFree(dk); return fail(c, SPEC_ENOMEM, "write_kv: staging"); }
    int rc = SPEC_OK;
    if (hipMemcpy(dk, k_host, count * 4, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(dv, v_host, count * 4, hipMemcpyHostToDevice) != hipSuccess ||
        launch_kv_write(kv_of(c, m, layer), m.s.dtype, seq, pos0, n, dk, dv, c->stream) != hipSuccess ||
        hipStreamSynchronize(c->stream) != hipSuccess)
        rc = fail(c, SPEC_EHIP, "write_kv: copy or launch failed");
    (void)hipFree(dk);
    (void)hipFree(dv);
    return rc;
}

int spec_profile_kernel(spec_ctx *c, int32_t model, int32_t kind) {
    if (!c) return SPEC_EINVAL;
    if (model != 0 && model != 1) return fail(c, SPEC_EINVAL, "profile: model must be 0 (draft) or 1 (target)");
    if (kind < -1 || kind > 7) return fail(c, SPEC_EINVAL, "profile: unknown kernel class");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->prof_epi = kind;
    c->prof_model = model;
    c->prof_used = 0;
    return SPEC_OK;
}

int spec_profile_read_class(spec_ctx *c, int32_t model, int32_t kind, int32_t *launches, double *total_ms) {
    if (!c || !launches || !total_ms) return fail(c, SPEC_EINVAL, "profile_read: null pointer");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    double tot = 0.0;
    int n = 0;
    for (size_t i = 0; i + 1 < c->prof_used; i += 2) {
        const int tag = c->prof_tag[i / 2];
        if (kind >= 0 && tag != 16 * model + kind) continue;
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, c->prof_events[i], c->prof_events[i + 1]));
        tot += ms;
        n += 1;
    }
    *launches = n;
    *total_ms = tot;
    return SPEC_OK;
}

int spec_profile_read(spec_ctx *c, int32_t *launches, double *total_ms) {
    const int rc = spec_profile_read_class(c, 0, -1, launches, total_ms);
    if (rc == SPEC_OK) c->prof_used = 0;
    return rc;
}

// ---- single kernels -------------------------------------------------------------------------------

int spec_k_gemv(const void *w, int32_t dtype, int32_t N, int32_t K, const float *x, int32_t R, float *y, int32_t path,
                void *stream) {
    if (!w || !x || !y || N < 1 || K < 1 || R < 1 || R > 128) return SPEC_EINVAL;
    if (dtype != SPEC_F32 && dtype != SPEC_BF16) return SPEC_EINVAL;
    if (K % (dtype == SPEC_BF16 ? 8 : 4)) return SPEC_EINVAL;
    GemvArgs a{};
    a.w0 = w; a.n0 = N; a.K = K; a.R = R; a.x = x; a.x_mul = 1; a.y = y;
    if (path == SPEC_PATH_MFMA) {
        // x is split into two bf16 terms in a scratch copy: the matrix-core kernel reads 16-bit rows
        if (dtype != SPEC_BF16 || N % 16 || K % 32) return SPEC_EINVAL;
        const hipStream_t st = reinterpret_cast<hipStream_t>(stream);
        // one block: the two bf16 terms of x, then the partial tiles and zeroed arrival counters of the kernel that
        // shares K out over workgroups
        uint16_t *xb = nullptr;
        const size_t x_bytes = ((size_t)R * K * 4 + 255) & ~(size_t)255;
        const size_t part_bytes = (size_t)KSPLIT_MAX * (N / 16) * 256 * sizeof(float), tick_bytes = KSPLIT_TICKETS * sizeof(uint32_t);
        if (hipMalloc(reinterpret_cast<void **>(&xb), x_bytes + part_bytes + tick_bytes) != hipSuccess) return SPEC_ENOMEM;
        int rc = SPEC_OK;
        uint8_t *blk = reinterpret_cast<uint8_t *>(xb);
        a.ks_part = reinterpret_cast<float *>(blk + x_bytes);
        a.ks_ticket = reinterpret_cast<uint32_t *>(blk + x_bytes + part_bytes);
        if (hipMemsetAsync(a.ks_ticket, 0, tick_bytes, st) != hipSuccess) rc = SPEC_EHIP;
        if (launch_cast_to_bf16(x, xb, (int64_t)R * K, (int64_t)R * K, st) != hipSuccess) rc = SPEC_EHIP;
        a.xb = xb; a.xb_lo = (int64_t)R * K;
        if (rc == SPEC_OK && launch_gemv_mfma(a, EPI_PLAIN, 0, nullptr, nullptr, st) != hipSuccess) rc = SPEC_EHIP;
        if (hipStreamSynchronize(st) != hipSuccess) rc = SPEC_EHIP;
        (void)hipFree(xb);
        return rc;
    }
    a.rpw = gemv_wavedot_uses_split(EPI_PLAIN, N, K, R, dtype) ? 0 : gemv_wavedot_pick_rpw(EPI_PLAIN, N, K, R, dtype);
    if (launch_gemv_wavedot(a, EPI_PLAIN, dtype, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) return SPEC_EHIP;
    return SPEC_OK;
}

int spec_k_gemv_tiled(const void *w_tiled, int32_t N, int32_t K, const void *x_bf16, const void *x_lo_bf16, int32_t R,
                      float *y, int32_t cfg, void *stream) {
    if (!w_tiled || !x_bf16 || !y || N < 16 || K < 32 || N % 16 || K % 32 || R < 1 || R > 128) return SPEC_EINVAL;
    if (cfg != 0) {
        const int ng = cfg / 100, nw = cfg % 100;
        const int mb = R <= 16 ? 1 : (R <= 32 ? 2 : (R <= 64 ? 4 : 8));
        const bool known = (ng == 1 && (nw == 16 || nw == 8 || nw == 4)) || (ng == 2 && (nw == 8 || nw == 4)) ||
                           (ng == 4 && nw == 4);
        if (!known || ng * nw * mb > 32) return SPEC_EINVAL;
    }
    GemvArgs a{};
    a.w0 = w_tiled; a.n0 = N; a.K = K; a.R = R; a.xb = reinterpret_cast<const uint16_t *>(x_bf16); a.x_mul = 1; a.y = y;
    if (x_lo_bf16) a.xb_lo = reinterpret_cast<const uint16_t *>(x_lo_bf16) - a.xb;
    const hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    return launch_gemv_mfma(a, EPI_PLAIN, cfg, nullptr, nullptr, st) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

int spec_k_gemm_tiled(const void *w_tiled, int32_t N, int32_t K, const float *x, int32_t R, float *y, int32_t cfg,
                      void *workspace, int64_t workspace_bytes, void *stream) {
    if (!w_tiled || !x || !y || N < 16 || K < 32 || N % 16 || K % 32 || R < 1 || workspace_bytes < 0) return SPEC_EINVAL;
    const int shape = cfg % 1000, shares = cfg / 1000;
    if (cfg < 0 || (shape != 0 && shape != 408 && shape != 404 && shape != 304 && shape != 204 && shape != 104 && shape != 808 && shape != 524) || shares > 8) return SPEC_EINVAL;
    GemvArgs a{};
    a.w0 = w_tiled; a.n0 = N; a.K = K; a.R = R; a.x = x; a.x_mul = 1; a.y = y;
    const hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const hipError_t e = launch_gemm_mfma(a, EPI_PLAIN, cfg, nullptr, reinterpret_cast<float *>(workspace),
                                          workspace ? (size_t)workspace_bytes : 0, nullptr, nullptr, st);
    return e == hipSuccess ? SPEC_OK : (e == hipErrorInvalidValue ? SPEC_EINVAL : SPEC_EHIP);
}

int spec_k_retile_q8(const void *w_q8, int32_t N, int32_t K, void *out, void *stream) {
    if (!w_q8 || !out || N < 16 || K < 64 || N % 16 || K % 64) return SPEC_EINVAL;
    RetileArgs ra{};
    ra.w0 = w_q8; ra.mode = EPI_PLAIN; ra.Ntot = N; ra.K = K; ra.q8 = 1;
    if (launch_retile(ra, out, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) return SPEC_EHIP;
    return SPEC_OK;
}

int spec_k_gemv_tiled_q8(const void *w_tiled, const float *w_scale, int32_t N, int32_t K, const void *x_bf16,
                         const void *x_lo_bf16, int32_t R, float *y, void *stream) {
    if (!w_tiled || !w_scale || !x_bf16 || !y || N < 16 || K < 64 || N % 16 || K % 64 || R < 1 || R > 128) return SPEC_EINVAL;
    GemvArgs a{};
    a.w0 = w_tiled; a.wscale = w_scale; a.n0 = N; a.K = K; a.R = R; a.xb = reinterpret_cast<const uint16_t *>(x_bf16);
    a.x_mul = 1; a.y = y;
    if (x_lo_bf16) a.xb_lo = reinterpret_cast<const uint16_t *>(x_lo_bf16) - a.xb;
    const hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    return launch_gemv_mfma(a, EPI_PLAIN, 0, nullptr, nullptr, st) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

int spec_k_gemm_tiled_q8(const void *w_tiled, const float *w_scale, int32_t N, int32_t K, const float *x, int32_t R,
                         float *y, int32_t cfg, void *workspace, int64_t workspace_bytes, void *stream) {
    if (!w_tiled || !w_scale || !x || !y || N < 16 || K < 64 || N % 16 || K % 64 || R < 1 || workspace_bytes < 0) return SPEC_EINVAL;
    const int shape = cfg % 1000, shares = cfg / 1000;
    if (cfg < 0 || (shape != 0 && shape != 408 && shape != 404 && shape != 304 && shape != 204 && shape != 104 && shape != 808) || shares > 8) return SPEC_EINVAL;
    GemvArgs a{};
    a.w0 = w_tiled; a.wscale = w_scale; a.n0 = N; a.K = K; a.R = R; a.x = x; a.x_mul = 1; a.y = y;
    const hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const hipError_t e = launch_gemm_mfma(a, EPI_PLAIN, cfg, nullptr, reinterpret_cast<float *>(workspace),
                                          workspace ? (size_t)workspace_bytes : 0, nullptr, nullptr, st);
    return e == hipSuccess ? SPEC_OK : (e == hipErrorInvalidValue ? SPEC_EINVAL : SPEC_EHIP);
}

int spec_k_retile(const void *w, int32_t N, int32_t K, void *out, void *stream) {
    if (!w || !out || N < 16 || K < 32 || N % 16 || K % 32) return SPEC_EINVAL;
    RetileArgs ra{};
    ra.w0 = w; ra.mode = EPI_PLAIN; ra.Ntot = N; ra.K = K;
    if (launch_retile(ra, out, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) return SPEC_EHIP;
    return SPEC_OK;
}

int spec_k_copy(void *dst, const void *src, int64_t bytes, void *stream) {
    if (!dst || !src || bytes < 0 || bytes % 16) return SPEC_EINVAL;
    if (launch_copy(src, dst, bytes, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) return SPEC_EHIP;
    return SPEC_OK;
}

int spec_k_philox(uint64_t seed, const uint32_t *ctr, int32_t n, uint32_t *out, void *stream) {
    if (!ctr || !out || n < 0) return SPEC_EINVAL;
    if (launch_philox(seed, ctr, n, out, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) return SPEC_EHIP;
    return SPEC_OK;
}

int spec_k_accept(const float *p_logits, const float *q_logits, const int32_t *drafted, int32_t k, int32_t vocab,
                  float temperature, uint64_t seed, int32_t step, int32_t *result, void *stream) {
    if (!p_logits || !q_logits || !drafted || !result || k < 1 || k > 64 || vocab < 2 || !(temperature >= 0.f))
        return SPEC_EINVAL;
    const hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const AcceptScratch L = accept_scratch_layout(k, vocab);
    uint8_t *buf = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&buf), L.total) != hipSuccess) return SPEC_ENOMEM;
    int rc = SPEC_OK;
    auto ok = [&](hipError_t e) { if (e != hipSuccess && rc == SPEC_OK) rc = SPEC_EHIP; return e == hipSuccess; };
    ok(hipMemsetAsync(buf, 0, L.total, st));
    int32_t *state = reinterpret_cast<int32_t *>(buf + L.o_state);
    const int32_t init[16] = {0, 0, k, k, step, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    ok(hipMemcpyAsync(state, init, sizeof(init), hipMemcpyHostToDevice, st));
    ok(hipStreamSynchronize(st));  // `init` lives on this stack frame
    ok(hipMemcpyAsync(buf + L.o_tok, drafted, sizeof(int32_t) * k, hipMemcpyDeviceToDevice, st));
    ok(accept_on_scratch(buf, L, p_logits, q_logits, drafted, k, vocab, temperature, seed, st));
    ok(hipMemcpyAsync(result, state + 12, sizeof(int32_t) * 2, hipMemcpyDeviceToDevice, st));
    ok(hipStreamSynchronize(st));
    (void)hipFree(buf);
    return rc;
}

int spec_k_accept_static(const float *p_logits, const float *q_logits, const int32_t *drafted, int32_t k, int32_t vocab,
                         float temperature, uint64_t seed, int32_t step, int32_t *result, void *stream) {
    if (!p_logits || !q_logits || !drafted || !result || k < 1 || !(temperature >= 0.f)) return fail(nullptr, SPEC_EINVAL, "accept_static: bad arguments");
    if (k > SPEC_ACCEPT_STATIC_MAX_K || vocab < 2 || vocab > SPEC_ACCEPT_STATIC_MAX_VOCAB)
        return fail(nullptr, SPEC_EINVAL, "accept_static: k beyond 64 or vocab beyond 262144: the fixed scratch array does not hold it");
    const AcceptScratch L = accept_scratch_layout(k, vocab);
    if (L.total > sizeof(g_accept_scratch)) return fail(nullptr, SPEC_EINVAL, "accept_static: scratch layout exceeds the fixed array");
    uint8_t *buf = nullptr;
    const int rc0 = accept_static_scratch(&buf);
    if (rc0 != SPEC_OK) return rc0;
    const hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // every call on this GPU shares the array, which still holds the last call's contents: clear what this call
    // uses, by a kernel (a caller may be capturing the stream into a graph), and set the step state
    const int n16 = (int)(L.total / 16);
    hipLaunchKernelGGL(accept_scratch_init_k, dim3((n16 + 255) / 256), dim3(256), 0, st, reinterpret_cast<uint4 *>(buf), n16,
                       reinterpret_cast<int32_t *>(buf + L.o_state), reinterpret_cast<int32_t *>(buf + L.o_tok), drafted,
                       (int)k, (int)step);
    if (hipGetLastError() != hipSuccess) return fail(nullptr, SPEC_EHIP, "accept_static: launch failed");
    if (accept_on_scratch(buf, L, p_logits, q_logits, drafted, k, vocab, temperature, seed, st) != hipSuccess)
        return fail(nullptr, SPEC_EHIP, "accept_static: launch failed");
    hipLaunchKernelGGL(accept_result_k, dim3(1), dim3(64), 0, st, reinterpret_cast<const int32_t *>(buf + L.o_state) + 12, result);
    if (hipGetLastError() != hipSuccess) return fail(nullptr, SPEC_EHIP, "accept_static: launch failed");
    return SPEC_OK;
}

}  // extern "C"
