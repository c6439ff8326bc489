/*
 * dkv.h - C boundary of the MI355X (gfx950) library for the delayed KV-cache (dKV-Cache) hot path
 * of masked diffusion language models (arxiv 2505.15781).
 *
 * The hot path is one denoising step: choose the rows to recompute, run the transformer on those
 * rows only, overwrite their K/V in a position-indexed cache, attend (unmasked) over all positions,
 * take the vocabulary softmax of the candidate rows and commit the most confident ones.
 *
 * Conventions
 *  - Every pointer is marked (dev) = device memory or (host) = host memory.
 *  - All device memory is owned by the caller (weights, cache, token state, logs, workspace) and
 *    must outlive the context. The library allocates only the small host-side context, and never
 *    device memory.
 *  - All device work is enqueued on the caller's HIP stream (a hipStream_t passed as void*); calls
 *    return without waiting for it, except the dkv_read_* debug calls and dkv_profile_end, which
 *    synchronise that stream.
 *  - Every call returns 0 on success or a negative DKV_E_* code; dkv_last_error() gives the text
 *    of the most recent failure on this thread. No call aborts or throws.
 *  - Positions are 0-based; the generated region is [prompt_len, prompt_len + gen_len).
 */
#ifndef DKV_H
#define DKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* storage / arithmetic type of weights, activations fed to the projections, and the K/V cache;
 * accumulation, softmax, the residual stream and confidences are always fp32 */
#define DKV_BF16 0
#define DKV_FP32 1

/* cache variants (Sec. 3.3 "dKV-Cache-Decode", "dKV-Cache-Prefill and dKV-Cache-PD"; Sec. 3.4) */
#define DKV_DECODE  0
#define DKV_GREEDY  1
#define DKV_PREFILL 2
#define DKV_PD      3

/* remasking (Sec. 3.1 "Sampling Process"): keep the most confident, or a predefined order */
#define DKV_CONFIDENCE   0
#define DKV_RANDOM_ORDER 1

/* centre of the Greedy local window (Sec. 3.4): the position decoded now, or one step ago */
#define DKV_CENTER_CUR  0
#define DKV_CENTER_PREV 1

/* scope of an explicit refresh */
#define DKV_SCOPE_ALL 0
#define DKV_SCOPE_GEN 1

#define DKV_OK                     0
#define DKV_E_INVALID_ARG         -1
#define DKV_E_BAD_STATE           -2
#define DKV_E_UNSUPPORTED         -3
#define DKV_E_WORKSPACE_TOO_SMALL -4
#define DKV_E_HIP                 -5

typedef struct dkv_ctx dkv_ctx;

/* Pre-norm transformer block without biases: RMSNorm, rotary embedding (half-split pairing
 * i <-> i + head_dim/2), bidirectional attention with n_q_heads / n_kv_heads query heads sharing
 * each K/V head, SwiGLU feed-forward. head_dim must be 32, 64 or 128 and even. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, mask_id;
    int32_t dtype;                     /* DKV_BF16 or DKV_FP32 */
    float rms_eps, rope_theta;
} dkv_model_desc;

/* Weights, all (dev), row-major [out_features, in_features] so that y = x * W^T, elements of
 * model dtype; norm gains are fp32 in both modes.
 *   embed, lm_head [vocab, d_model]; final_norm [d_model]
 *   wqkv[l]      [(n_q_heads + 2 n_kv_heads) * head_dim, d_model]: Q rows (head-major), K rows, V rows
 *   wo[l]        [d_model, n_q_heads * head_dim]
 *   w_gate_up[l] [2 * d_ffn, d_model]: row 2j is gate_j, row 2j+1 is up_j
 *   w_down[l]    [d_model, d_ffn]
 *   norm1[l], norm2[l] [d_model]
 * The six per-layer members are (host) arrays of n_layers (dev) pointers; the arrays themselves
 * are copied during dkv_init_cache and need not outlive it. */
typedef struct {
    const void *embed, *lm_head;
    const float *final_norm;
    const void *const *wqkv, *const *wo, *const *w_gate_up, *const *w_down;
    const float *const *norm1, *const *norm2;
} dkv_weights;

/* The run: sequence, step schedule, refresh interval and variant.
 * Requirements (else DKV_E_INVALID_ARG): gen_len % block_len == 0; steps % (gen_len / block_len)
 * == 0; block_len % steps_per_block == 0 (k = block_len / steps_per_block positions are
 * committed per step per sequence); refresh_interval >= 1. Step 0 always recomputes everything;
 * afterwards step t is a scheduled refresh iff t % refresh_interval == 0 (Sec. 3.3, "Cache
 * Refreshing Mechanism"). */
typedef struct {
    int32_t batch, prompt_len, gen_len, steps, block_len, refresh_interval;
    int32_t variant;                   /* DKV_DECODE | DKV_GREEDY | DKV_PREFILL | DKV_PD */
    int32_t delay;                     /* 1: recompute the previous step's commits once more before
                                          caching them (Eq. 4); 0: cache at once (Eq. 3) */
    int32_t window, window_center, include_prev;   /* Greedy: window size w, its centre, and whether
                                                      the previous step's commits are recomputed */
    int32_t remask;                    /* DKV_CONFIDENCE | DKV_RANDOM_ORDER */
    int32_t shift_logits;              /* 0: the output at position q is the distribution of token q;
                                          1: of token q + 1 (models adapted from autoregressive ones,
                                          Appendix B, K/V cached unshifted): the row before every
                                          position that may be committed joins the active set and
                                          supplies its logits. Needs prompt_len >= 1. */
    const int32_t *order;              /* (dev) [batch, gen_len] absolute positions in commit order;
                                          DKV_RANDOM_ORDER only (required by DKV_GREEDY) */
} dkv_run_desc;

/* Caller-owned device state. k_cache / v_cache hold post-rotation keys and values of every
 * position: [n_layers][batch][n_kv_heads][seq_len][head_dim], model dtype, seq_len = prompt_len +
 * gen_len. tokens must hold the prompt ids in [:, :prompt_len] before dkv_init_cache.
 * decoded_* are logs of what each step committed, [steps][batch][k]. */
typedef struct {
    void *k_cache, *v_cache;           /* (dev) */
    int32_t *tokens;                   /* (dev) [batch, seq_len], in/out */
    uint8_t *masked;                   /* (dev) [batch, seq_len], 1 = not yet finalised */
    int32_t *stamp;                    /* (dev) [batch, seq_len], last step that wrote K/V; -1 never */
    int32_t *decoded_pos, *decoded_tok;/* (dev) [steps, batch, k] */
    float *decoded_conf;               /* (dev) [steps, batch, k] */
    void *workspace;                   /* (dev) scratch, 256-byte aligned */
    size_t workspace_bytes;
} dkv_buffers;

/* Bytes of workspace dkv_init_cache needs for this model and run (0 on invalid descriptors). */
size_t dkv_workspace_bytes(const dkv_model_desc *model, const dkv_run_desc *run);

/* Bind buffers and start a run: generated region of tokens := mask_id, masked := [p >= prompt_len],
 * stamp := -1, logs cleared, step counter := 0 (state before the first step of Sec. 3.1's sampling
 * process). The descriptors are copied. `stream` is a hipStream_t. */
int dkv_init_cache(dkv_ctx **out, const dkv_model_desc *model, const dkv_weights *weights,
                   const dkv_run_desc *run, const dkv_buffers *buffers, void *stream);

/* Compute the active set A_t of step `step` on the device (Eq. 4: everything still masked plus the
 * previous step's commits; all positions, or the generated region, on a refresh; the Greedy set
 * of Sec. 3.4). Rows are ordered sequence by sequence, position ascending.
 * active_idx (dev, nullable) receives the positions and must have room for batch * seq_len entries:
 * the call copies as many entries as the schedule's bound below says, which is not known before the
 * call and can exceed the true row count; entries from active_off[batch] on are undefined.
 * active_off (dev, nullable) [batch+1] receives the row offsets of each sequence.
 * host_upper_bound_rows (host, nullable) receives a bound on the row count known from the schedule
 * without reading the device (exact except for Greedy, whose windows may clip or overlap, and for
 * shifted logits). `step` must be the context's next step, else DKV_E_BAD_STATE.
 * Calling it is optional: dkv_denoise_step does it when it has not been done for that step. */
int dkv_select_active(dkv_ctx *ctx, int32_t step, int32_t *active_idx, int32_t *active_off,
                      int32_t *host_upper_bound_rows);

/* One denoising step (Algorithm 1 plus the unmasking of Sec. 3.1): embed the active rows, per
 * layer project Q/K/V, rotate, overwrite the rows' K/V in the cache, attend over all positions,
 * output projection, feed-forward; then final norm, vocabulary logits, softmax confidence and
 * arg max (MASK excluded, lowest id on ties) for the candidate rows (active, masked, in the
 * current block), and commit k positions per sequence: the most confident (ties to the lower
 * position) or the next entries of `order`.
 * forced_pos / forced_tok (dev, nullable, [batch, k]): commit these instead (teacher forcing);
 * each forced position must be a candidate of the step. logits_out (dev, nullable) receives the
 * fp32 logits of the candidate rows, [n_candidates, vocab], candidates ordered like the rows.
 * `step` must be the context's next step; the counter advances by one. */
int dkv_denoise_step(dkv_ctx *ctx, int32_t step, const int32_t *forced_pos,
                     const int32_t *forced_tok, float *logits_out);

/* Make the next step recompute the given scope whatever the schedule says (the cache refresh of
 * Sec. 3.3 on demand; also the way to rebuild a cache from tokens and mask alone). */
int dkv_refresh(dkv_ctx *ctx, int32_t scope);

/* Debug reads; each synchronises the stream. Sizes are capacities of the (host) outputs.
 * dkv_read_rows: active set of the last selected step: positions and offsets [batch+1].
 * dkv_read_candidates: candidates of the last executed step: position, predicted token,
 *   confidence, and offsets [batch+1].
 * dkv_read_hidden: the residual stream of the last executed step, [rows, d_model] fp32, at a layer
 *   boundary: `layer` = l in [0, n_layers) is the input of block l (l = 0: the embedded rows), `layer` =
 *   n_layers the output of the last block (before the final norm). The input of block l together with
 *   the cache rows of layer l is everything one block of Algorithm 1 (lines 3-6) consumes, so a single
 *   layer can be checked on its own at any step. Only `layer` = n_layers is kept by default; the other
 *   boundaries are available when dkv_capture_hidden was active during the step, else
 *   DKV_E_BAD_STATE. */
int dkv_read_rows(dkv_ctx *ctx, int32_t *pos, int32_t *off, int32_t capacity, int32_t *n_rows);
int dkv_read_candidates(dkv_ctx *ctx, int32_t *pos, int32_t *tok, float *conf, int32_t *off,
                        int32_t capacity, int32_t *n_cand);
int dkv_read_hidden(dkv_ctx *ctx, int32_t layer, float *out, int32_t capacity_rows, int32_t *n_rows);

/* Debug: from the next step on, every denoising step also copies the residual stream at each layer
 * boundary into `buffer` (dev), laid out [n_layers + 1][batch * seq_len][d_model] fp32 (slot l = input
 * of block l, slot n_layers = output of the last block; only the step's rows of each slot are written).
 * `bytes` is the buffer's size: DKV_E_INVALID_ARG if smaller than that layout. buffer = NULL stops the
 * copies. The buffer is caller-owned and must stay valid while capturing. */
int dkv_capture_hidden(dkv_ctx *ctx, float *buffer, size_t bytes);

int dkv_destroy(dkv_ctx *ctx);

/* Per-kernel timing for roofline reports. Between dkv_profile_begin and dkv_profile_end every
 * launch of a projection or attention kernel made by dkv_denoise_step is bracketed by HIP events on
 * the context's stream. dkv_profile_end synchronises the stream and fills `out` (host, array of
 * DKV_PROF_KINDS entries) with, per kernel kind: number of launches, summed duration in
 * milliseconds, and summed algorithmic bytes and flops of those launches:
 *   projection  bytes = (M*K + N*K) * sizeof(element) + output bytes   flops = 2*M*N*K
 *               (output: 4*M*N; M*(N/2)*sizeof(element) for gate/up with the fused SwiGLU; 0 for the
 *               vocabulary projection, whose epilogue keeps the softmax statistics only)
 *   attention   bytes = (2*batch*n_kv_heads*seq_len + 2*rows*n_q_heads) * head_dim * sizeof(element)
 *               flops = 4*rows*n_q_heads*seq_len*head_dim
 * with M the schedule's row count of the step. Kinds: */
#define DKV_GEMM_DMA_32x128   0   /* projection kernels by workgroup tile (rows x columns) */
#define DKV_GEMM_DMA_64x128   1
#define DKV_GEMM_DMA_128x128  2
#define DKV_GEMM_DMA_128x256  3
#define DKV_GEMM_DMA_256x256  4
#define DKV_GEMM_DMA_128x96   5
#define DKV_GEMM_DMA_128x192  6
#define DKV_GEMM_DMA_256x192  7
#define DKV_GEMM_DMA_192x256  8
#define DKV_GEMM_REG_64x128   9   /* bf16 with K not a multiple of 64 */
#define DKV_GEMM_SIMT         10  /* fp32 mode / generic */
#define DKV_PROF_ATTN         11  /* attention (including the key-slice merge when it runs) */
#define DKV_PROF_KINDS        12
typedef struct {
    int64_t launches;
    double ms, bytes, flops;
} dkv_prof_entry;
int dkv_profile_begin(dkv_ctx *ctx);
int dkv_profile_end(dkv_ctx *ctx, dkv_prof_entry *out);

/* Text of the last error raised on the calling thread ("" if none). Never NULL. */
const char *dkv_last_error(void);

/* The cache update and attention of one layer in isolation (Algorithm 1 lines 4-6 in a
 * position-indexed layout; Eq. 4): for every active row r of sequence b at position
 * p = active_idx[r], k_cache[b][:, p, :] = k_new[r], v_cache[b][:, p, :] = v_new[r]; then
 * out[r, h, :] = softmax(q[r, h] . K[b][h / group]^T / sqrt(head_dim)) V[b][h / group] over ALL
 * seq_len positions, no mask.
 * All (dev): k_cache, v_cache [batch][n_kv_heads][seq_len][head_dim]; q, out [rows][n_q_heads]
 * [head_dim]; k_new, v_new [rows][n_kv_heads][head_dim]; active_idx [rows] (positions, distinct
 * within a sequence); active_off [batch+1]. `rows` (host) = active_off[batch];
 * `max_rows_per_seq` (host) bounds the rows of any one sequence (pass `rows` if unknown). Elements
 * of `dtype`. workspace (dev) of dkv_attn_update_workspace_bytes(...) bytes for the same bound. */
size_t dkv_attn_update_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                       int32_t seq_len, int32_t head_dim, int32_t dtype,
                                       int32_t max_rows_per_seq);
int dkv_attn_update(void *k_cache, void *v_cache, const void *q, const void *k_new,
                    const void *v_new, const int32_t *active_idx, const int32_t *active_off,
                    void *out, int32_t rows, int32_t max_rows_per_seq, int32_t batch,
                    int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len, int32_t head_dim,
                    int32_t dtype, void *workspace, size_t workspace_bytes, void *stream);

/* dkv_attn_update for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, same kernels and the same
 * result as dkv_attn_update, but the scratch of key-sliced attention (partial softmax records) is a
 * DKV_STATIC_SCRATCH_BYTES array inside the library's device image; the call allocates nothing. Shapes whose
 * scratch (dkv_attn_update_workspace_bytes) exceeds that size get DKV_E_WORKSPACE_TOO_SMALL and nothing is
 * launched. Each GPU holds one such array for the life of the process and all calls on that GPU share it:
 * calls that overlap on one GPU (different streams or threads) race on it; calls on one stream are ordered.
 * Nothing in the array needs clearing between calls. The first call on a device looks the array up and must
 * not happen inside a graph capture. */
#define DKV_STATIC_SCRATCH_BYTES (4u << 20)
int dkv_attn_update_static(void *k_cache, void *v_cache, const void *q, const void *k_new,
                           const void *v_new, const int32_t *active_idx, const int32_t *active_off,
                           void *out, int32_t rows, int32_t max_rows_per_seq, int32_t batch,
                           int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len, int32_t head_dim,
                           int32_t dtype, void *stream);

/* The paper's own cache operator, concat_reorder (Appendix A; Algorithm 1 lines 4-5), on its compact
 * layout: per (sequence, kv head) the n_cached cached rows and the n_new freshly computed rows are
 * concatenated and row i of the result is row take[b][i] of that concatenation (the order that puts the next
 * step's cached positions first). Not on this library's path (the position-indexed cache never moves);
 * exported so that what the layout choice saves can be measured on the same shapes.
 * All (dev): k_cached, v_cached [batch][n_kv_heads][n_cached][head_dim]; k_new, v_new [batch][n_kv_heads]
 * [n_new][head_dim]; take [batch][n_cached + n_new], a permutation of 0 .. n_cached + n_new - 1 per
 * sequence (values are not checked); k_out, v_out [batch][n_kv_heads][n_cached + n_new][head_dim], must not
 * overlap the inputs. head_dim * element size must be a multiple of 16. */
int dkv_concat_reorder(const void *k_cached, const void *v_cached, const void *k_new, const void *v_new,
                       const int32_t *take, void *k_out, void *v_out, int32_t batch, int32_t n_kv_heads,
                       int32_t n_cached, int32_t n_new, int32_t head_dim, int32_t dtype, void *stream);

/* y[M, N] (fp32, dev) = x[M, K] * w[N, K]^T with x, w of `dtype` (dev): the projection kernel of
 * the path on its own, for parity tests and roofline measurements. workspace as returned by
 * dkv_gemm_workspace_bytes. */
size_t dkv_gemm_workspace_bytes(int32_t m, int32_t n, int32_t k, int32_t dtype);
int dkv_gemm(const void *x, const void *w, float *y, int32_t m, int32_t n, int32_t k,
             int32_t dtype, void *workspace, size_t workspace_bytes, void *stream);
/* The same with the kernel (DKV_GEMM_*), the number of K slices and the launch options chosen by the
 * caller instead of the library's heuristic, so every kernel can be checked on every shape. workspace
 * must hold split_k * m * n floats when split_k > 1. `options` is a sum of DKV_GEMM_OPT_* (ignored by
 * the kernels that have no such option, and dropped when the grid does not fit them).
 * DKV_E_UNSUPPORTED if the kernel does not take the shape, DKV_E_INVALID_ARG for unknown option bits. */
#define DKV_GEMM_OPT_STAGGER    1   /* every workgroup starts its K loop at a different K tile */
#define DKV_GEMM_OPT_XCD_GROUP  2   /* workgroups that share an XCD's L2 take neighbouring tiles */
#define DKV_GEMM_OPT_STREAM_W   8   /* weights fetched with the non-temporal hint (dropped with more than one row of tiles) */
#define DKV_GEMM_OPT_SWIGLU     4   /* fused SwiGLU epilogue: w rows are gate_0, up_0, gate_1, up_1, ...; y is then
                                       a `dtype` (bf16) array [M, N/2] with y[m][j] = silu(x w_{2j}) * (x w_{2j+1});
                                       tile kernels with split_k == 1 only, else DKV_E_UNSUPPORTED */
int dkv_gemm_with(const void *x, const void *w, void *y, int32_t m, int32_t n, int32_t k,
                  int32_t dtype, int32_t kind, int32_t split_k, int32_t options, void *workspace,
                  size_t workspace_bytes, void *stream);

/* Yardsticks for roofline reports, not part of the path: what the chip sustains for a plain copy (the kernel
 * HBM byte counters are calibrated with), a streaming read, and a register-only dense bf16 MFMA loop. All
 * (dev) buffers; `bytes` a multiple of 16; sink: at least 2 MiB, never written in practice. dkv_peak_mfma stores
 * the flops of its launch in *flops (host). The caller times the launches on `stream`. */
int dkv_peak_copy(const void *src, void *dst, size_t bytes, void *stream);
int dkv_peak_read(const void *src, void *sink, size_t bytes, void *stream);
int dkv_peak_mfma(void *sink, int32_t iters, double *flops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DKV_H */
