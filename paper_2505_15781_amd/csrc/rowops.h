// Launchers of the row-wise and index kernels (see rowops.hip).
#pragma once
#include "common.h"

enum { SEL_ALL = 0, SEL_GEN = 1, SEL_MASKED_PREV = 2, SEL_GREEDY = 3 };
enum { STATUS_NAN = 1, STATUS_BAD_COMMIT = 2 };

struct SelectArgs {
    const uint8_t *masked;   // [batch][L]
    const int *d_prev;       // [batch][k], -1 = none
    const int *order;        // [batch][G] or null
    int *row_pos, *row_seq;  // [rows]
    int *row_off;            // [batch+1]
    int *cand_row, *cand_pos;// [cands]
    int *cand_off;           // [batch+1]
    int *counts;             // [0] rows, [1] candidates
    int batch, L, P, G, k, step;
    int mode, use_prev, center_prev, window, win_lo, win_hi;
    int blk_lo, blk_hi;
    int shift;               // 1: a candidate's prediction is the output of the row before it
};

struct CommitArgs {
    const int *cand_off, *cand_pos, *cand_tok;
    const float *cand_conf;
    uint8_t *taken;
    const int *forced_pos, *forced_tok, *order;
    int *tokens;
    uint8_t *masked;
    int *d_prev;
    int *log_pos, *log_tok;
    float *log_conf;
    int *status;
    int batch, L, G, k, step;
};

int dkv_launch_select(const SelectArgs &a, hipStream_t s);
int dkv_launch_embed_norm(int dtype, hipStream_t s, int rows, int d, const void *embed, const int *tokens,
                          const int *row_pos, const int *row_seq, const int *counts, const float *gain,
                          float *h, void *a, int *stamp, int L, float eps, int step);
int dkv_launch_residual_norm(int dtype, hipStream_t s, int rows, int d, const float *part, int splits,
                             size_t stride, const int *counts, const float *gain, float *h, void *a,
                             float eps);
int dkv_launch_rope_scatter(int dtype, hipStream_t s, int rows, const float *part, int splits, size_t stride,
                            const int *row_pos, const int *row_seq, const int *counts, const float *rope,
                            void *q, void *Kc, void *Vc, int Hq, int Hkv, int dh, int L);
int dkv_launch_swiglu(int dtype, hipStream_t s, int rows, const float *part, int splits, size_t stride,
                      const int *counts, void *f, int F);
int dkv_launch_gather_rows(int dtype, hipStream_t s, int cands, const void *src, const int *cand_row,
                           const int *counts, void *dst, int d);
int dkv_launch_reduce_partials(hipStream_t s, const float *part, int splits, size_t stride, float *out,
                               size_t total);
constexpr int HEAD_SLICES = 16;     // vocabulary ranges per candidate row in the head statistics
size_t dkv_head_stats_scratch_bytes(int cands);
int dkv_launch_head_stats(hipStream_t s, int cands, const float *logits, const int *counts, int V,
                          int mask_id, int *tok, float *conf, int *status, void *scratch);
// merge of the per-column-tile records that the vocabulary projection's epilogue leaves: [cands][n_part]
int dkv_launch_head_merge(hipStream_t s, int cands, const void *head_part, int n_part, const int *counts, int *tok,
                          float *conf, int *status);
int dkv_launch_commit(const CommitArgs &a, hipStream_t s);
int dkv_launch_init_state(hipStream_t s, int *tokens, uint8_t *masked, int *stamp, int *d_prev, int *status,
                          int batch, int L, int P, int k, int mask_id);
// table[p][i] = (cos, sin)(p * theta^(-2 i / dh)), i < dh / 2, evaluated in double precision
int dkv_launch_rope_table(hipStream_t s, float *table, int L, int dh, double theta);
int dkv_launch_fill_i32(hipStream_t s, int *p, int v, size_t n);
int dkv_launch_fill_u8(hipStream_t s, uint8_t *p, uint8_t v, size_t n);
int dkv_launch_concat_reorder(hipStream_t s, const void *k_cached, const void *v_cached, const void *k_new,
                              const void *v_new, const int *take, void *k_out, void *v_out, int batch, int heads,
                              int n_cached, int n_new, int row_bytes);
int dkv_launch_scatter_rows(int dtype, hipStream_t s, int rows, const void *k_new, const void *v_new,
                            const int *idx, const int *off, void *Kc, void *Vc, int batch, int Hkv, int L,
                            int dh);
