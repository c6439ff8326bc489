// C boundary: context, workspace layout, and the per-step kernel sequence.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"
#include "rowops.h"

static thread_local char g_err[512] = "";

void dkv_set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

extern "C" const char *dkv_last_error(void) { return g_err; }

namespace {

bool run_ok(const dkv_run_desc &r) {
    if (r.batch < 1 || r.prompt_len < 0 || r.gen_len < 1 || r.steps < 1 || r.block_len < 1 ||
        r.refresh_interval < 1)
        return false;
    if (r.gen_len % r.block_len) return false;
    const int nb = r.gen_len / r.block_len;
    if (r.steps % nb) return false;
    const int spb = r.steps / nb;
    if (r.block_len % spb) return false;
    if (r.variant < DKV_DECODE || r.variant > DKV_PD) return false;
    if (r.remask != DKV_CONFIDENCE && r.remask != DKV_RANDOM_ORDER) return false;
    if (r.variant == DKV_GREEDY && r.remask != DKV_RANDOM_ORDER) return false;
    if (r.window < 0 || (r.delay != 0 && r.delay != 1)) return false;
    if (r.shift_logits != 0 && (r.shift_logits != 1 || r.prompt_len < 1)) return false;
    return true;
}

bool model_ok(const dkv_model_desc &m) {
    if (m.n_layers < 1 || m.d_model < 1 || m.n_q_heads < 1 || m.n_kv_heads < 1 || m.d_ffn < 1 || m.vocab < 2)
        return false;
    if (m.n_q_heads % m.n_kv_heads) return false;
    if (m.head_dim != 32 && m.head_dim != 64 && m.head_dim != 128) return false;
    if (m.mask_id < 0 || m.mask_id >= m.vocab) return false;
    if (m.dtype != DKV_BF16 && m.dtype != DKV_FP32) return false;
    if (m.d_model > 8192 || m.d_model % 4 || m.d_ffn % 2) return false;
    return true;
}

struct Layout {
    size_t rope, row_pos, row_seq, row_off, cand_row, cand_pos, cand_off, counts, cand_tok, cand_conf, taken,
        d_prev, status, h, a, q, attn_out, f, a_c, logits, part, attn_part, total;
    size_t head_part;
    size_t part_floats, attn_part_bytes;
    int rows_cap, cand_cap;
    size_t head_records;   // most (candidate row, column tile) records a vocabulary projection leaves
    bool head_fused;       // softmax statistics leave the vocabulary projection's epilogue: no fp32 logits buffer
};

Layout make_layout(const dkv_model_desc &m, const dkv_run_desc &r) {
    Layout y;
    const int L = r.prompt_len + r.gen_len, B = r.batch;
    const int nb = r.gen_len / r.block_len, spb = r.steps / nb, k = r.block_len / spb;
    const size_t es = m.dtype == DKV_BF16 ? 2 : 4;
    y.rows_cap = B * L;
    y.cand_cap = B * r.block_len;
    const int qn = m.n_q_heads * m.head_dim, nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    // partial-sum buffer: worst case over every row count a step can have
    size_t pf = 0;
    for (int rows = 1; rows <= y.rows_cap; ++rows) {
        GemmPlan p1 = dkv_gemm_plan(m.dtype, rows, nqkv, m.d_model);
        GemmPlan p2 = dkv_gemm_plan(m.dtype, rows, m.d_model, qn);
        GemmPlan p3 = dkv_gemm_plan(m.dtype, rows, 2 * m.d_ffn, m.d_model);
        GemmPlan p4 = dkv_gemm_plan(m.dtype, rows, m.d_model, m.d_ffn);
        size_t a = (size_t)p1.split_k * rows * nqkv, b = (size_t)p2.split_k * rows * m.d_model,
               c = (size_t)p3.split_k * rows * 2 * m.d_ffn, d = (size_t)p4.split_k * rows * m.d_model;
        if (dkv_gemm_can_fuse_swiglu(m.dtype, 2 * m.d_ffn, m.d_model, p3)) c = 0;   // SwiGLU in the epilogue: no fp32 product
        if (a > pf) pf = a;
        if (b > pf) pf = b;
        if (c > pf) pf = c;
        if (d > pf) pf = d;
    }
    y.head_fused = true;
    y.head_records = 1;
    for (int c = 1; c <= y.cand_cap; ++c) {
        GemmPlan p = dkv_gemm_plan(m.dtype, c, m.vocab, m.d_model);
        if (p.split_k > 1) {
            size_t a = (size_t)p.split_k * c * m.vocab;
            if (a > pf) pf = a;
        }
        // the epilogue needs the tile kernel with one K slice for every candidate count of the run
        if (!dkv_gemm_can_fuse_head(m.dtype, m.d_model, p)) y.head_fused = false;
        else if ((size_t)c * dkv_gemm_tiles_n(p, m.vocab) > y.head_records) y.head_records = (size_t)c * dkv_gemm_tiles_n(p, m.vocab);
    }
    y.part_floats = pf;
    size_t ap = 0;
    for (int rows = 1; rows <= L; ++rows) {
        AttnPlan p = dkv_attn_plan(m.dtype, B, m.n_q_heads, m.n_kv_heads, L, m.head_dim, rows);
        size_t a = dkv_attn_partial_bytes(p, B, m.n_q_heads, m.n_kv_heads, m.head_dim);
        if (a > ap) ap = a;
    }
    y.attn_part_bytes = ap;

    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes, 256);
        return at;
    };
    y.rope = take((size_t)L * (m.head_dim / 2) * sizeof(float2));
    y.row_pos = take((size_t)y.rows_cap * 4);
    y.row_seq = take((size_t)y.rows_cap * 4);
    y.row_off = take((size_t)(B + 1) * 4);
    y.cand_row = take((size_t)y.cand_cap * 4);
    y.cand_pos = take((size_t)y.cand_cap * 4);
    y.cand_off = take((size_t)(B + 1) * 4);
    y.counts = take(16);
    y.cand_tok = take((size_t)y.cand_cap * 4);
    y.cand_conf = take((size_t)y.cand_cap * 4);
    y.taken = take((size_t)y.cand_cap);
    y.d_prev = take((size_t)B * k * 4);
    y.status = take(16);
    y.h = take((size_t)y.rows_cap * m.d_model * 4);
    y.a = take((size_t)y.rows_cap * m.d_model * es);
    y.q = take((size_t)y.rows_cap * qn * es);
    y.attn_out = take((size_t)y.rows_cap * qn * es);
    y.f = take((size_t)y.rows_cap * m.d_ffn * es);
    y.a_c = take((size_t)y.cand_cap * m.d_model * es);
    // fp32 logits of the candidate rows: only when the head's statistics cannot leave the projection's epilogue
    // (a caller who wants the logits passes a buffer of their own)
    y.logits = take(y.head_fused ? 0 : (size_t)y.cand_cap * m.vocab * 4);
    y.head_part = take(y.head_fused ? y.head_records * sizeof(HeadPartial)
                                    : dkv_head_stats_scratch_bytes(y.cand_cap));
    y.part = take(y.part_floats * 4);
    y.attn_part = take(y.attn_part_bytes);
    y.total = o;
    return y;
}

}  // namespace

struct dkv_ctx {
    dkv_model_desc m;
    dkv_run_desc r;
    dkv_buffers buf;
    hipStream_t stream;
    std::vector<const void *> wqkv, wo, wgu, wdown;
    std::vector<const float *> n1, n2;
    const void *embed, *lm_head;
    const float *final_norm;
    Layout lay;
    int L, k, spb;
    size_t es;
    // workspace views
    float2 *rope;
    int *row_pos, *row_seq, *row_off, *cand_row, *cand_pos, *cand_off, *counts, *cand_tok, *d_prev, *status;
    float *cand_conf, *h, *logits, *part;
    uint8_t *taken;
    void *a, *q, *attn_out, *f, *a_c, *attn_part, *head_part;
    // step state (host)
    int next_step, selected_step, forced_scope;
    int rows_upper, rows_per_seq_upper, cand_upper;
    int last_rows_upper, last_cand_upper;
    // optional copies of the residual stream at every layer boundary (debug)
    float *capture = nullptr;
    bool last_step_captured = false;
    // optional per-launch timing
    bool prof_on = false;
    struct ProfRec { hipEvent_t a, b; int kind; double bytes, flops; };
    std::vector<ProfRec> prof;
    std::vector<hipEvent_t> ev_pool;
};

namespace {

hipEvent_t prof_event(dkv_ctx *c) {
    hipEvent_t e = nullptr;
    if (!c->ev_pool.empty()) { e = c->ev_pool.back(); c->ev_pool.pop_back(); return e; }
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Brackets the launches made by `fn` with events when profiling is on.
template <typename F> int timed(dkv_ctx *c, int kind, double bytes, double flops, F fn) {
    if (!c->prof_on) return fn();
    hipEvent_t a = prof_event(c), b = prof_event(c);
    if (!a || !b) { dkv_set_error("hipEventCreate failed"); return DKV_E_HIP; }
    DKV_HIP_TRY(hipEventRecord(a, c->stream));
    int rc = fn();
    DKV_HIP_TRY(hipEventRecord(b, c->stream));
    c->prof.push_back({a, b, kind, bytes, flops});
    return rc;
}

int timed_gemm(dkv_ctx *c, const void *A, const void *W, float *out, int m, const int *m_dev, int n, int k,
               GemmPlan p) {
    const double es = (double)c->es;
    // output bytes: fp32 [M, N], or the fused SwiGLU's [M, N/2] elements
    const double out_bytes = (p.flags & GEMM_FLAG_SWIGLU) ? es * m * (n / 2) : 4.0 * m * n;
    return timed(c, p.kind, ((double)m * k + (double)n * k) * es + out_bytes,
                 2.0 * m * n * k,
                 [&] { return dkv_launch_gemm(c->m.dtype, A, W, out, m, m, m_dev, n, k, p, c->stream); });
}

template <typename P> P *ws(const dkv_ctx *c, size_t off) {
    return reinterpret_cast<P *>(static_cast<char *>(c->buf.workspace) + off);
}

// Row and candidate bounds of step t that follow from the schedule alone.
void step_bounds(const dkv_ctx *c, int t, int scope, int *mode, int *rows_per_seq, int *cand_per_seq) {
    const dkv_run_desc &r = c->r;
    const int L = c->L, G = r.gen_len, k = c->k;
    int md, rows;
    const bool refresh = (t % r.refresh_interval) == 0;
    if (scope == DKV_SCOPE_ALL) { md = SEL_ALL; rows = L; }
    else if (scope == DKV_SCOPE_GEN) { md = SEL_GEN; rows = G; }
    else if (t == 0) { md = SEL_ALL; rows = L; }
    else if (r.variant == DKV_PREFILL) { md = SEL_GEN; rows = G; }
    else if (refresh) {
        if (r.variant == DKV_PD) { md = SEL_GEN; rows = G; }
        else { md = SEL_ALL; rows = L; }
    } else if (r.variant == DKV_GREEDY) {
        md = SEL_GREEDY;
        rows = k * (r.window + 3);
        if (rows > L) rows = L;
    } else {
        md = SEL_MASKED_PREV;
        rows = G - t * k + (r.delay ? k : 0);
    }
    const int in_block = r.block_len - (t % c->spb) * k;
    const int cands = in_block < rows ? in_block : rows;
    // shifted logits: every candidate may pull the row before it into the set
    if (r.shift_logits && md != SEL_ALL) rows = rows + cands < L ? rows + cands : L;
    *mode = md;
    *rows_per_seq = rows;
    *cand_per_seq = cands;
}

int do_select(dkv_ctx *c, int step) {
    int mode, rps, cps;
    step_bounds(c, step, c->forced_scope, &mode, &rps, &cps);
    const dkv_run_desc &r = c->r;
    SelectArgs a;
    a.masked = c->buf.masked;
    a.d_prev = c->d_prev;
    a.order = r.order;
    a.row_pos = c->row_pos; a.row_seq = c->row_seq; a.row_off = c->row_off;
    a.cand_row = c->cand_row; a.cand_pos = c->cand_pos; a.cand_off = c->cand_off;
    a.counts = c->counts;
    a.batch = r.batch; a.L = c->L; a.P = r.prompt_len; a.G = r.gen_len; a.k = c->k; a.step = step;
    a.mode = mode;
    a.use_prev = (mode == SEL_GREEDY) ? r.include_prev : r.delay;
    a.center_prev = r.window_center == DKV_CENTER_PREV;
    a.window = r.window;
    a.win_lo = (r.window + 1) / 2;     // ceil(w/2) below the centre
    a.win_hi = r.window / 2;           // floor(w/2) above it
    const int j = step / c->spb;
    a.blk_lo = r.prompt_len + j * r.block_len;
    a.blk_hi = a.blk_lo + r.block_len;
    a.shift = r.shift_logits;
    int rc = dkv_launch_select(a, c->stream);
    if (rc) return rc;
    c->rows_per_seq_upper = rps;
    c->rows_upper = rps * r.batch;
    c->cand_upper = cps * r.batch;
    c->selected_step = step;
    c->forced_scope = -1;
    return DKV_OK;
}

}  // namespace

extern "C" size_t dkv_workspace_bytes(const dkv_model_desc *model, const dkv_run_desc *run) {
    if (!model || !run || !model_ok(*model) || !run_ok(*run)) return 0;
    return make_layout(*model, *run).total;
}

extern "C" int dkv_init_cache(dkv_ctx **out, const dkv_model_desc *model, const dkv_weights *w,
                              const dkv_run_desc *run, const dkv_buffers *buf, void *stream) {
    if (!out || !model || !w || !run || !buf) { dkv_set_error("null argument"); return DKV_E_INVALID_ARG; }
    if (!model_ok(*model)) { dkv_set_error("unsupported or inconsistent model descriptor"); return DKV_E_INVALID_ARG; }
    if (!run_ok(*run)) { dkv_set_error("schedule must tile: gen_len %% block_len, steps %% blocks, block_len %% steps_per_block, refresh_interval >= 1; Greedy needs a predefined order"); return DKV_E_INVALID_ARG; }
    if (run->remask == DKV_RANDOM_ORDER && !run->order) { dkv_set_error("RANDOM_ORDER needs run.order"); return DKV_E_INVALID_ARG; }
    if (!buf->k_cache || !buf->v_cache || !buf->tokens || !buf->masked || !buf->stamp || !buf->decoded_pos ||
        !buf->decoded_tok || !buf->decoded_conf || !buf->workspace) {
        dkv_set_error("null buffer"); return DKV_E_INVALID_ARG;
    }
    if (!w->embed || !w->lm_head || !w->final_norm || !w->wqkv || !w->wo || !w->w_gate_up || !w->w_down ||
        !w->norm1 || !w->norm2) { dkv_set_error("null weight pointer"); return DKV_E_INVALID_ARG; }
    if (reinterpret_cast<uintptr_t>(buf->workspace) % 256) { dkv_set_error("workspace must be 256-byte aligned"); return DKV_E_INVALID_ARG; }
    Layout lay = make_layout(*model, *run);
    if (buf->workspace_bytes < lay.total) {
        dkv_set_error("workspace has %zu bytes, %zu needed", buf->workspace_bytes, lay.total);
        return DKV_E_WORKSPACE_TOO_SMALL;
    }
    dkv_ctx *c = new (std::nothrow) dkv_ctx();
    if (!c) { dkv_set_error("out of host memory"); return DKV_E_INVALID_ARG; }
    c->m = *model; c->r = *run; c->buf = *buf; c->stream = static_cast<hipStream_t>(stream);
    for (int l = 0; l < model->n_layers; ++l) {
        if (!w->wqkv[l] || !w->wo[l] || !w->w_gate_up[l] || !w->w_down[l] || !w->norm1[l] || !w->norm2[l]) {
            delete c; dkv_set_error("null weight pointer in layer %d", l); return DKV_E_INVALID_ARG;
        }
        c->wqkv.push_back(w->wqkv[l]); c->wo.push_back(w->wo[l]); c->wgu.push_back(w->w_gate_up[l]);
        c->wdown.push_back(w->w_down[l]); c->n1.push_back(w->norm1[l]); c->n2.push_back(w->norm2[l]);
    }
    c->embed = w->embed; c->lm_head = w->lm_head; c->final_norm = w->final_norm;
    c->lay = lay;
    c->L = run->prompt_len + run->gen_len;
    c->spb = run->steps / (run->gen_len / run->block_len);
    c->k = run->block_len / c->spb;
    c->es = model->dtype == DKV_BF16 ? 2 : 4;
    c->rope = ws<float2>(c, lay.rope);
    c->row_pos = ws<int>(c, lay.row_pos); c->row_seq = ws<int>(c, lay.row_seq); c->row_off = ws<int>(c, lay.row_off);
    c->cand_row = ws<int>(c, lay.cand_row); c->cand_pos = ws<int>(c, lay.cand_pos); c->cand_off = ws<int>(c, lay.cand_off);
    c->counts = ws<int>(c, lay.counts); c->cand_tok = ws<int>(c, lay.cand_tok); c->cand_conf = ws<float>(c, lay.cand_conf);
    c->taken = ws<uint8_t>(c, lay.taken); c->d_prev = ws<int>(c, lay.d_prev); c->status = ws<int>(c, lay.status);
    c->h = ws<float>(c, lay.h); c->a = ws<void>(c, lay.a); c->q = ws<void>(c, lay.q);
    c->attn_out = ws<void>(c, lay.attn_out); c->f = ws<void>(c, lay.f); c->a_c = ws<void>(c, lay.a_c);
    c->logits = ws<float>(c, lay.logits); c->part = ws<float>(c, lay.part); c->attn_part = ws<void>(c, lay.attn_part);
    c->head_part = ws<void>(c, lay.head_part);
    c->next_step = 0; c->selected_step = -1; c->forced_scope = -1;
    c->rows_upper = c->cand_upper = c->last_rows_upper = c->last_cand_upper = 0;

    // rotary table (cos, sin) per (position, pair), computed in double precision and stored as fp32
    int rc = dkv_launch_rope_table(c->stream, reinterpret_cast<float *>(c->rope), c->L, model->head_dim,
                                   (double)model->rope_theta);
    if (rc) { delete c; return rc; }
    rc = dkv_launch_init_state(c->stream, buf->tokens, buf->masked, buf->stamp, c->d_prev, c->status,
                                   run->batch, c->L, run->prompt_len, c->k, model->mask_id);
    const size_t nlog = (size_t)run->steps * run->batch * c->k;
    if (!rc) rc = dkv_launch_fill_i32(c->stream, buf->decoded_pos, -1, nlog);
    if (!rc) rc = dkv_launch_fill_i32(c->stream, buf->decoded_tok, -1, nlog);
    if (!rc) rc = dkv_launch_fill_i32(c->stream, reinterpret_cast<int *>(buf->decoded_conf), 0, nlog);
    if (rc) { delete c; return rc; }
    *out = c;
    return DKV_OK;
}

extern "C" int dkv_select_active(dkv_ctx *c, int32_t step, int32_t *active_idx, int32_t *active_off,
                                 int32_t *host_upper_bound_rows) {
    if (!c) { dkv_set_error("null context"); return DKV_E_INVALID_ARG; }
    if (step != c->next_step || step >= c->r.steps) {
        dkv_set_error("select_active(step=%d) but the next step is %d of %d", step, c->next_step, c->r.steps);
        return DKV_E_BAD_STATE;
    }
    if (c->selected_step != step) {
        int rc = do_select(c, step);
        if (rc) return rc;
    }
    if (active_idx)   // the schedule's bound of entries; those past the true count are stale
        DKV_HIP_TRY(hipMemcpyAsync(active_idx, c->row_pos, (size_t)c->rows_upper * 4, hipMemcpyDeviceToDevice, c->stream));
    if (active_off)
        DKV_HIP_TRY(hipMemcpyAsync(active_off, c->row_off, (size_t)(c->r.batch + 1) * 4, hipMemcpyDeviceToDevice, c->stream));
    if (host_upper_bound_rows) *host_upper_bound_rows = c->rows_upper;
    return DKV_OK;
}

extern "C" int dkv_refresh(dkv_ctx *c, int32_t scope) {
    if (!c) { dkv_set_error("null context"); return DKV_E_INVALID_ARG; }
    if (scope != DKV_SCOPE_ALL && scope != DKV_SCOPE_GEN) { dkv_set_error("unknown refresh scope %d", scope); return DKV_E_INVALID_ARG; }
    c->forced_scope = scope;
    c->selected_step = -1;       // a selection already made for the next step is redone
    return DKV_OK;
}

extern "C" int dkv_denoise_step(dkv_ctx *c, int32_t step, const int32_t *forced_pos, const int32_t *forced_tok,
                                float *logits_out) {
    if (!c) { dkv_set_error("null context"); return DKV_E_INVALID_ARG; }
    if (step != c->next_step || step >= c->r.steps) {
        dkv_set_error("denoise_step(step=%d) but the next step is %d of %d", step, c->next_step, c->r.steps);
        return DKV_E_BAD_STATE;
    }
    if ((forced_pos == nullptr) != (forced_tok == nullptr)) { dkv_set_error("forced_pos and forced_tok go together"); return DKV_E_INVALID_ARG; }
    int rc;
    if (c->selected_step != step && (rc = do_select(c, step))) return rc;

    const dkv_model_desc &m = c->m;
    const dkv_run_desc &r = c->r;
    hipStream_t s = c->stream;
    const int rows = c->rows_upper, cands = c->cand_upper, d = m.d_model, dt = m.dtype;
    const int qn = m.n_q_heads * m.head_dim, nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    const int *n_rows = c->counts, *n_cand = c->counts + 1;
    const size_t layer_elems = (size_t)r.batch * m.n_kv_heads * c->L * m.head_dim;

    if ((rc = dkv_launch_embed_norm(dt, s, rows, d, c->embed, c->buf.tokens, c->row_pos, c->row_seq, c->counts,
                                    c->n1[0], c->h, c->a, c->buf.stamp, c->L, m.rms_eps, step))) return rc;
    const AttnPlan ap = dkv_attn_plan(dt, r.batch, m.n_q_heads, m.n_kv_heads, c->L, m.head_dim, c->rows_per_seq_upper);
    const size_t slot_floats = (size_t)c->lay.rows_cap * d;
    auto capture = [&](int slot) -> int {
        if (!c->capture || rows <= 0) return DKV_OK;
        DKV_HIP_TRY(hipMemcpyAsync(c->capture + slot * slot_floats, c->h, (size_t)rows * d * 4,
                                   hipMemcpyDeviceToDevice, s));
        return DKV_OK;
    };
    for (int l = 0; l < m.n_layers; ++l) {
        if ((rc = capture(l))) return rc;
        char *Kl = static_cast<char *>(c->buf.k_cache) + layer_elems * c->es * l;
        char *Vl = static_cast<char *>(c->buf.v_cache) + layer_elems * c->es * l;
        GemmPlan p = dkv_gemm_plan(dt, rows, nqkv, d);
        if ((rc = timed_gemm(c, c->a, c->wqkv[l], c->part, rows, n_rows, nqkv, d, p))) return rc;
        if ((rc = dkv_launch_rope_scatter(dt, s, rows, c->part, p.split_k, (size_t)rows * nqkv, c->row_pos, c->row_seq,
                                          c->counts, reinterpret_cast<const float *>(c->rope), c->q, Kl, Vl,
                                          m.n_q_heads, m.n_kv_heads, m.head_dim, c->L))) return rc;
        rc = timed(c, DKV_PROF_ATTN,
                   (2.0 * r.batch * m.n_kv_heads * c->L + 2.0 * rows * m.n_q_heads) * m.head_dim * (double)c->es,
                   4.0 * rows * m.n_q_heads * (double)c->L * m.head_dim, [&] {
                       return dkv_launch_attention(dt, c->q, Kl, Vl, c->row_off, c->attn_out, r.batch, m.n_q_heads,
                                                   m.n_kv_heads, c->L, m.head_dim, rows, ap, c->attn_part,
                                                   AttnFusedUpdate{nullptr, nullptr, nullptr}, s);
                   });
        if (rc) return rc;
        p = dkv_gemm_plan(dt, rows, d, qn);
        if ((rc = timed_gemm(c, c->attn_out, c->wo[l], c->part, rows, n_rows, d, qn, p))) return rc;
        if ((rc = dkv_launch_residual_norm(dt, s, rows, d, c->part, p.split_k, (size_t)rows * d, c->counts, c->n2[l],
                                           c->h, c->a, m.rms_eps))) return rc;
        p = dkv_gemm_plan(dt, rows, 2 * m.d_ffn, d);
        if (dkv_gemm_can_fuse_swiglu(dt, 2 * m.d_ffn, d, p)) {
            // single K slice: SwiGLU in the projection's epilogue, the fp32 gate/up product is never written
            p.flags |= GEMM_FLAG_SWIGLU;
            if ((rc = timed_gemm(c, c->a, c->wgu[l], reinterpret_cast<float *>(c->f), rows, n_rows, 2 * m.d_ffn, d, p))) return rc;
        } else {
            if ((rc = timed_gemm(c, c->a, c->wgu[l], c->part, rows, n_rows, 2 * m.d_ffn, d, p))) return rc;
            if ((rc = dkv_launch_swiglu(dt, s, rows, c->part, p.split_k, (size_t)rows * 2 * m.d_ffn, c->counts, c->f, m.d_ffn))) return rc;
        }
        p = dkv_gemm_plan(dt, rows, d, m.d_ffn);
        if ((rc = timed_gemm(c, c->f, c->wdown[l], c->part, rows, n_rows, d, m.d_ffn, p))) return rc;
        const float *next_gain = (l + 1 < m.n_layers) ? c->n1[l + 1] : c->final_norm;
        if ((rc = dkv_launch_residual_norm(dt, s, rows, d, c->part, p.split_k, (size_t)rows * d, c->counts, next_gain,
                                           c->h, c->a, m.rms_eps))) return rc;
    }
    if ((rc = capture(m.n_layers))) return rc;
    c->last_step_captured = c->capture != nullptr;
    // vocabulary head on the candidate rows only (same result as projecting every active row)
    if ((rc = dkv_launch_gather_rows(dt, s, cands, c->a, c->cand_row, c->counts, c->a_c, d))) return rc;
    GemmPlan hp = dkv_gemm_plan(dt, cands, m.vocab, d);
    if (c->lay.head_fused) {
        // softmax maximum, sum and arg max per column tile leave the projection's epilogue and a small kernel merges
        // the tiles of a row: the [candidates, vocab] logits are never written (unless the caller asks for them)
        GemmEpilogue eh;
        eh.kind = EPI_HEAD;
        eh.out = logits_out;
        eh.head_part = static_cast<HeadPartial *>(c->head_part);
        eh.head_tiles = dkv_gemm_tiles_n(hp, m.vocab);
        eh.mask_id = m.mask_id;
        eh.status = c->status;
        rc = timed(c, hp.kind, ((double)cands * d + (double)m.vocab * d) * (double)c->es + (logits_out ? 4.0 * cands * m.vocab : 0.0),
                   2.0 * cands * m.vocab * d,
                   [&] { return dkv_launch_gemm_head(c->a_c, c->lm_head, cands, n_cand, m.vocab, d, hp, eh, s); });
        if (rc) return rc;
        if ((rc = dkv_launch_head_merge(s, cands, c->head_part, eh.head_tiles, c->counts, c->cand_tok, c->cand_conf, c->status))) return rc;
    } else {
        float *lg = logits_out ? logits_out : c->logits;
        if (hp.split_k == 1) {
            if ((rc = timed_gemm(c, c->a_c, c->lm_head, lg, cands, n_cand, m.vocab, d, hp))) return rc;
        } else {
            if ((rc = timed_gemm(c, c->a_c, c->lm_head, c->part, cands, n_cand, m.vocab, d, hp))) return rc;
            if ((rc = dkv_launch_reduce_partials(s, c->part, hp.split_k, (size_t)cands * m.vocab, lg, (size_t)cands * m.vocab))) return rc;
        }
        if ((rc = dkv_launch_head_stats(s, cands, lg, c->counts, m.vocab, m.mask_id, c->cand_tok, c->cand_conf, c->status,
                                        c->head_part))) return rc;
    }

    CommitArgs ca;
    ca.cand_off = c->cand_off; ca.cand_pos = c->cand_pos; ca.cand_tok = c->cand_tok; ca.cand_conf = c->cand_conf;
    ca.taken = c->taken; ca.forced_pos = forced_pos; ca.forced_tok = forced_tok;
    ca.order = (r.remask == DKV_RANDOM_ORDER) ? r.order : nullptr;
    ca.tokens = c->buf.tokens; ca.masked = c->buf.masked; ca.d_prev = c->d_prev;
    ca.log_pos = c->buf.decoded_pos; ca.log_tok = c->buf.decoded_tok; ca.log_conf = c->buf.decoded_conf;
    ca.status = c->status;
    ca.batch = r.batch; ca.L = c->L; ca.G = r.gen_len; ca.k = c->k; ca.step = step;
    if ((rc = dkv_launch_commit(ca, s))) return rc;

    c->last_rows_upper = rows;
    c->last_cand_upper = cands;
    c->next_step = step + 1;
    return DKV_OK;
}

namespace {
int check_status(dkv_ctx *c) {
    int st = 0;
    DKV_HIP_TRY(hipMemcpyAsync(&st, c->status, 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipStreamSynchronize(c->stream));
    if (st & STATUS_NAN) { dkv_set_error("NaN logits were produced"); return DKV_E_BAD_STATE; }
    if (st & STATUS_BAD_COMMIT) { dkv_set_error("a step could not commit: forced or ordered position was not a candidate"); return DKV_E_BAD_STATE; }
    return DKV_OK;
}
}  // namespace

extern "C" int dkv_read_rows(dkv_ctx *c, int32_t *pos, int32_t *off, int32_t capacity, int32_t *n_rows) {
    if (!c || !pos || !off || !n_rows) { dkv_set_error("null argument"); return DKV_E_INVALID_ARG; }
    if (c->selected_step < 0) { dkv_set_error("no step has been selected yet"); return DKV_E_BAD_STATE; }
    std::vector<int> o(c->r.batch + 1);
    DKV_HIP_TRY(hipMemcpyAsync(o.data(), c->row_off, o.size() * 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipStreamSynchronize(c->stream));
    const int n = o.back();
    if (n > capacity || n > c->lay.rows_cap) { dkv_set_error("%d rows do not fit capacity %d", n, capacity); return DKV_E_INVALID_ARG; }
    memcpy(off, o.data(), o.size() * 4);
    DKV_HIP_TRY(hipMemcpyAsync(pos, c->row_pos, (size_t)n * 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipStreamSynchronize(c->stream));
    *n_rows = n;
    return DKV_OK;
}

extern "C" int dkv_read_candidates(dkv_ctx *c, int32_t *pos, int32_t *tok, float *conf, int32_t *off,
                                   int32_t capacity, int32_t *n_cand) {
    if (!c || !pos || !tok || !conf || !off || !n_cand) { dkv_set_error("null argument"); return DKV_E_INVALID_ARG; }
    if (c->next_step == 0) { dkv_set_error("no step has been executed yet"); return DKV_E_BAD_STATE; }
    int rc = check_status(c);
    if (rc) return rc;
    std::vector<int> o(c->r.batch + 1);
    DKV_HIP_TRY(hipMemcpyAsync(o.data(), c->cand_off, o.size() * 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipStreamSynchronize(c->stream));
    const int n = o.back();
    if (n > capacity || n > c->lay.cand_cap) { dkv_set_error("%d candidates do not fit capacity %d", n, capacity); return DKV_E_INVALID_ARG; }
    if (n > c->last_cand_upper) { dkv_set_error("%d candidates exceed the schedule's bound %d", n, c->last_cand_upper); return DKV_E_BAD_STATE; }
    memcpy(off, o.data(), o.size() * 4);
    DKV_HIP_TRY(hipMemcpyAsync(pos, c->cand_pos, (size_t)n * 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipMemcpyAsync(tok, c->cand_tok, (size_t)n * 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipMemcpyAsync(conf, c->cand_conf, (size_t)n * 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipStreamSynchronize(c->stream));
    *n_cand = n;
    return DKV_OK;
}

extern "C" int dkv_read_hidden(dkv_ctx *c, int32_t layer, float *out, int32_t capacity_rows, int32_t *n_rows) {
    if (!c || !out || !n_rows) { dkv_set_error("null argument"); return DKV_E_INVALID_ARG; }
    if (layer < 0 || layer > c->m.n_layers) { dkv_set_error("layer boundary %d outside 0..%d", layer, c->m.n_layers); return DKV_E_INVALID_ARG; }
    if (c->next_step == 0) { dkv_set_error("no step has been executed yet"); return DKV_E_BAD_STATE; }
    if (layer != c->m.n_layers && !c->last_step_captured) {
        dkv_set_error("layer boundary %d was not kept: dkv_capture_hidden was not active during the last step", layer);
        return DKV_E_BAD_STATE;
    }
    int n = 0;
    DKV_HIP_TRY(hipMemcpyAsync(&n, c->counts, 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipStreamSynchronize(c->stream));
    if (n > capacity_rows) { dkv_set_error("%d rows do not fit capacity %d", n, capacity_rows); return DKV_E_INVALID_ARG; }
    if (n > c->last_rows_upper) { dkv_set_error("%d rows exceed the schedule's bound %d", n, c->last_rows_upper); return DKV_E_BAD_STATE; }
    const float *src = layer == c->m.n_layers ? c->h : c->capture + (size_t)layer * c->lay.rows_cap * c->m.d_model;
    DKV_HIP_TRY(hipMemcpyAsync(out, src, (size_t)n * c->m.d_model * 4, hipMemcpyDeviceToHost, c->stream));
    DKV_HIP_TRY(hipStreamSynchronize(c->stream));
    *n_rows = n;
    return DKV_OK;
}

extern "C" int dkv_capture_hidden(dkv_ctx *c, float *buffer, size_t bytes) {
    if (!c) { dkv_set_error("null context"); return DKV_E_INVALID_ARG; }
    const size_t need = (size_t)(c->m.n_layers + 1) * c->lay.rows_cap * c->m.d_model * sizeof(float);
    if (buffer && bytes < need) { dkv_set_error("capture buffer has %zu bytes, %zu needed", bytes, need); return DKV_E_INVALID_ARG; }
    c->capture = buffer;
    return DKV_OK;
}

extern "C" int dkv_profile_begin(dkv_ctx *c) {
    if (!c) { dkv_set_error("null context"); return DKV_E_INVALID_ARG; }
    for (auto &r : c->prof) { c->ev_pool.push_back(r.a); c->ev_pool.push_back(r.b); }
    c->prof.clear();
    c->prof_on = true;
    return DKV_OK;
}

extern "C" int dkv_profile_end(dkv_ctx *c, dkv_prof_entry *out) {
    if (!c || !out) { dkv_set_error("null argument"); return DKV_E_INVALID_ARG; }
    if (!c->prof_on) { dkv_set_error("profiling was not started"); return DKV_E_BAD_STATE; }
    c->prof_on = false;
    DKV_HIP_TRY(hipStreamSynchronize(c->stream));
    for (int i = 0; i < DKV_PROF_KINDS; ++i) out[i] = dkv_prof_entry{0, 0.0, 0.0, 0.0};
    for (auto &r : c->prof) {
        float ms = 0.f;
        DKV_HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
        out[r.kind].launches += 1;
        out[r.kind].ms += ms;
        out[r.kind].bytes += r.bytes;
        out[r.kind].flops += r.flops;
        c->ev_pool.push_back(r.a);
        c->ev_pool.push_back(r.b);
    }
    c->prof.clear();
    return DKV_OK;
}

extern "C" int dkv_destroy(dkv_ctx *c) {
    if (c) {
        for (auto &r : c->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (auto e : c->ev_pool) (void)hipEventDestroy(e);
    }
    delete c;
    return DKV_OK;
}

// ------------------------------------------------------------------------------ isolated entry points

extern "C" size_t dkv_attn_update_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                                  int32_t seq_len, int32_t head_dim, int32_t dtype,
                                                  int32_t max_rows_per_seq) {
    if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || seq_len < 1 || max_rows_per_seq < 0)
        return 0;
    AttnPlan p = dkv_attn_plan(dtype, batch, n_q_heads, n_kv_heads, seq_len, head_dim, max_rows_per_seq);
    return align_up(dkv_attn_partial_bytes(p, batch, n_q_heads, n_kv_heads, head_dim) + 256, 256);
}

namespace {
int attn_update_impl(void *k_cache, void *v_cache, const void *q, const void *k_new, const void *v_new,
                     const int32_t *active_idx, const int32_t *active_off, void *out, int32_t rows,
                     int32_t max_rows_per_seq, int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                     int32_t seq_len, int32_t head_dim, int32_t dtype, void *workspace, size_t workspace_bytes,
                     const char *workspace_name, void *stream) {
    if (!k_cache || !v_cache || !active_off) { dkv_set_error("null argument"); return DKV_E_INVALID_ARG; }
    if (rows < 0 || batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || seq_len < 1 ||
        max_rows_per_seq < 0 || max_rows_per_seq > seq_len || rows > (long)batch * max_rows_per_seq) {
        dkv_set_error("inconsistent sizes"); return DKV_E_INVALID_ARG;
    }
    if (head_dim != 32 && head_dim != 64 && head_dim != 128) { dkv_set_error("head_dim %d not supported (32, 64, 128)", head_dim); return DKV_E_UNSUPPORTED; }
    if (dtype != DKV_BF16 && dtype != DKV_FP32) { dkv_set_error("unknown dtype"); return DKV_E_INVALID_ARG; }
    if (rows == 0) return DKV_OK;
    if (!q || !k_new || !v_new || !active_idx || !out) { dkv_set_error("null argument"); return DKV_E_INVALID_ARG; }
    AttnPlan p = dkv_attn_plan(dtype, batch, n_q_heads, n_kv_heads, seq_len, head_dim, max_rows_per_seq);
    size_t need = dkv_attn_partial_bytes(p, batch, n_q_heads, n_kv_heads, head_dim);
    if (need > workspace_bytes || (need && !workspace)) {
        dkv_set_error("%s has %zu bytes, %zu needed", workspace_name, workspace_bytes, need);
        return DKV_E_WORKSPACE_TOO_SMALL;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // few rows per sequence: the attention kernel writes the new rows into the cache itself
    if (dkv_attn_can_fuse_update(p, max_rows_per_seq))
        return dkv_launch_attention(dtype, q, k_cache, v_cache, active_off, out, batch, n_q_heads, n_kv_heads,
                                    seq_len, head_dim, rows, p, workspace, AttnFusedUpdate{k_new, v_new, active_idx}, s);
    int rc = dkv_launch_scatter_rows(dtype, s, rows, k_new, v_new, active_idx, active_off, k_cache, v_cache, batch,
                                     n_kv_heads, seq_len, head_dim);
    if (rc) return rc;
    return dkv_launch_attention(dtype, q, k_cache, v_cache, active_off, out, batch, n_q_heads, n_kv_heads, seq_len,
                                head_dim, rows, p, workspace, AttnFusedUpdate{nullptr, nullptr, nullptr}, s);
}
}  // namespace

extern "C" int dkv_attn_update(void *k_cache, void *v_cache, const void *q, const void *k_new, const void *v_new,
                               const int32_t *active_idx, const int32_t *active_off, void *out, int32_t rows,
                               int32_t max_rows_per_seq, int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                               int32_t seq_len, int32_t head_dim, int32_t dtype, void *workspace,
                               size_t workspace_bytes, void *stream) {
    return attn_update_impl(k_cache, v_cache, q, k_new, v_new, active_idx, active_off, out, rows, max_rows_per_seq,
                            batch, n_q_heads, n_kv_heads, seq_len, head_dim, dtype, workspace, workspace_bytes,
                            "workspace", stream);
}

// ---- the same operation for callers that cannot allocate ------------------------------------------------
// The partial (max, sum, output) records of key-sliced attention live in a device array that is part of the
// library's image: every GPU the library runs on holds its own copy for the life of the process.
static __device__ __align__(256) unsigned char scratch[DKV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};        // device address of `scratch` on each device, looked up once

// Device address of this GPU's copy of `scratch` (the array's name is only a host-side handle).
int static_scratch(void **ptr) {
    int dev = -1;
    DKV_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { dkv_set_error("device ordinal %d not supported", dev); return DKV_E_UNSUPPORTED; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        DKV_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { dkv_set_error("hipGetSymbolAddress returned a null address"); return DKV_E_HIP; }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return DKV_OK;
}
}  // namespace

extern "C" int dkv_attn_update_static(void *k_cache, void *v_cache, const void *q, const void *k_new,
                                      const void *v_new, const int32_t *active_idx, const int32_t *active_off,
                                      void *out, int32_t rows, int32_t max_rows_per_seq, int32_t batch,
                                      int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len, int32_t head_dim,
                                      int32_t dtype, void *stream) {
    void *ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc) return rc;
    // Every record the merge kernel reads is written by the attention kernel of the same call, so nothing in
    // the array has to start at zero; contents left by an earlier (larger) call are never read.
    return attn_update_impl(k_cache, v_cache, q, k_new, v_new, active_idx, active_off, out, rows, max_rows_per_seq,
                            batch, n_q_heads, n_kv_heads, seq_len, head_dim, dtype, ws, DKV_STATIC_SCRATCH_BYTES,
                            "the library's static scratch array", stream);
}

extern "C" int dkv_concat_reorder(const void *k_cached, const void *v_cached, const void *k_new, const void *v_new,
                                  const int32_t *take, void *k_out, void *v_out, int32_t batch, int32_t n_kv_heads,
                                  int32_t n_cached, int32_t n_new, int32_t head_dim, int32_t dtype, void *stream) {
    if (batch < 1 || n_kv_heads < 1 || n_cached < 0 || n_new < 0 || head_dim < 1 ||
        (dtype != DKV_BF16 && dtype != DKV_FP32)) { dkv_set_error("bad argument"); return DKV_E_INVALID_ARG; }
    if (n_cached + n_new == 0) return DKV_OK;
    if (!take || !k_out || !v_out || (n_cached && (!k_cached || !v_cached)) || (n_new && (!k_new || !v_new))) {
        dkv_set_error("null argument"); return DKV_E_INVALID_ARG;
    }
    const int row_bytes = head_dim * (dtype == DKV_BF16 ? 2 : 4);
    if (row_bytes % 16) { dkv_set_error("a row of head_dim %d elements is not a multiple of 16 bytes", head_dim); return DKV_E_UNSUPPORTED; }
    return dkv_launch_concat_reorder(static_cast<hipStream_t>(stream), k_cached, v_cached, k_new, v_new, take, k_out,
                                     v_out, batch, n_kv_heads, n_cached, n_new, row_bytes);
}

extern "C" size_t dkv_gemm_workspace_bytes(int32_t m, int32_t n, int32_t k, int32_t dtype) {
    if (m < 1 || n < 1 || k < 1) return 0;
    GemmPlan p = dkv_gemm_plan(dtype, m, n, k);
    return p.split_k > 1 ? (size_t)p.split_k * m * n * 4 : 0;
}

extern "C" int dkv_gemm_with(const void *x, const void *w, void *yv, int32_t m, int32_t n, int32_t k, int32_t dtype,
                             int32_t kind, int32_t split_k, int32_t options, void *workspace,
                             size_t workspace_bytes, void *stream) {
    float *y = static_cast<float *>(yv);
    if (!x || !w || !y || m < 1 || n < 1 || k < 1) { dkv_set_error("bad argument"); return DKV_E_INVALID_ARG; }
    if (options & ~(DKV_GEMM_OPT_STAGGER | DKV_GEMM_OPT_XCD_GROUP | DKV_GEMM_OPT_SWIGLU | DKV_GEMM_OPT_STREAM_W)) {
        dkv_set_error("unknown projection option bits 0x%x", options);
        return DKV_E_INVALID_ARG;
    }
    if (dtype != DKV_BF16 && dtype != DKV_FP32) { dkv_set_error("unknown dtype"); return DKV_E_INVALID_ARG; }
    GemmPlan p;
    p.kind = kind;
    p.split_k = split_k < 0 ? 2 : split_k;
    p.frac_units = split_k < 0 ? (k / 64) * 3 / 4 : 0;      // split_k = -1 asks for the 3/4 share
    p.flags = ((options & DKV_GEMM_OPT_STAGGER) ? GEMM_FLAG_STAGGER : 0) |
              ((options & DKV_GEMM_OPT_XCD_GROUP) ? GEMM_FLAG_XCD_GROUP : 0) |
              ((options & DKV_GEMM_OPT_STREAM_W) ? GEMM_FLAG_STREAM_W : 0);
    if (options & DKV_GEMM_OPT_SWIGLU) {
        if (!dkv_gemm_can_fuse_swiglu(dtype, n, k, p)) {
            dkv_set_error("kernel %d with %d K slices cannot fuse SwiGLU (bf16 tile kernels, one K slice, even N)", kind, split_k);
            return DKV_E_UNSUPPORTED;
        }
        p.flags |= GEMM_FLAG_SWIGLU;
    }
    if (!dkv_gemm_plan_valid(dtype, k, p)) {
        dkv_set_error("kernel %d with %d K slices does not take dtype %d, K %d", kind, split_k, dtype, k);
        return DKV_E_UNSUPPORTED;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (p.split_k == 1) return dkv_launch_gemm(dtype, x, w, y, m, m, nullptr, n, k, p, s);
    size_t need = (size_t)p.split_k * m * n * 4;
    if (!workspace || workspace_bytes < need) {
        dkv_set_error("workspace has %zu bytes, %zu needed", workspace_bytes, need);
        return DKV_E_WORKSPACE_TOO_SMALL;
    }
    int rc = dkv_launch_gemm(dtype, x, w, static_cast<float *>(workspace), m, m, nullptr, n, k, p, s);
    if (rc) return rc;
    return dkv_launch_reduce_partials(s, static_cast<const float *>(workspace), p.split_k, (size_t)m * n, y,
                                      (size_t)m * n);
}

extern "C" int dkv_gemm(const void *x, const void *w, float *y, int32_t m, int32_t n, int32_t k, int32_t dtype,
                        void *workspace, size_t workspace_bytes, void *stream) {
    if (m < 1 || n < 1 || k < 1) { dkv_set_error("bad argument"); return DKV_E_INVALID_ARG; }
    GemmPlan p = dkv_gemm_plan(dtype, m, n, k);
    const int options = ((p.flags & GEMM_FLAG_STAGGER) ? DKV_GEMM_OPT_STAGGER : 0) |
                        ((p.flags & GEMM_FLAG_XCD_GROUP) ? DKV_GEMM_OPT_XCD_GROUP : 0) |
                        ((p.flags & GEMM_FLAG_STREAM_W) ? DKV_GEMM_OPT_STREAM_W : 0);
    return dkv_gemm_with(x, w, y, m, n, k, dtype, p.kind, p.split_k, options, workspace, workspace_bytes, stream);
}
