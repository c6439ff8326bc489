// Row-wise and index kernels of one denoising step: active-set selection, embedding gather, RMSNorm,
// rotary embedding + K/V scatter into the position-indexed cache, SwiGLU, vocabulary softmax
// statistics, and the confidence top-k commit.
#include "rowops.h"

namespace {

// ------------------------------------------------------------------------------------------------
// Active set (Eq. 4; Sec. 3.3 refresh / Prefill / PD; Sec. 3.4 Greedy). One workgroup walks the
// sequences in order and compacts the flagged positions with a block-wide prefix sum, so rows come
// out sequence by sequence, position ascending.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int block_excl_scan(int v, int *wave_tot, int *total) {
    // exclusive prefix sum over the block (1024 threads); returns the prefix, *total the sum
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    int x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int y = __shfl_up(x, o, 64);
        if (lane >= o) x += y;
    }
    __syncthreads();
    if (lane == 63) wave_tot[w] = x;
    __syncthreads();
    int base = 0, tot = 0;
    for (int i = 0; i < nw; ++i) {
        int t = wave_tot[i];
        if (i < w) base += t;
        tot += t;
    }
    *total = tot;
    return base + x - v;
}

__global__ __launch_bounds__(1024) void select_active_kernel(SelectArgs a) {
    __shared__ int wave_tot[16];
    int row_base = 0, cand_base = 0;
    for (int b = 0; b < a.batch; ++b) {
        if (threadIdx.x == 0) {
            a.row_off[b] = row_base;
            a.cand_off[b] = cand_base;
        }
        const uint8_t *mk = a.masked + (size_t)b * a.L;
        for (int p0 = 0; p0 < a.L; p0 += blockDim.x) {
            const int p = p0 + threadIdx.x;
            int act = 0, cand = 0;
            if (p < a.L) {
                // membership of position x in the variant's set, and whether x may be committed at this step
                auto in_set = [&](int x) -> bool {
                    if (a.mode == SEL_ALL) return true;
                    if (a.mode == SEL_GEN) return x >= a.P;
                    if (a.mode == SEL_MASKED_PREV) {
                        bool f = mk[x] != 0;
                        if (!f && a.use_prev)
                            for (int j = 0; j < a.k; ++j) f |= (a.d_prev[b * a.k + j] == x);
                        return f;
                    }
                    bool f = false;   // SEL_GREEDY
                    for (int j = 0; j < a.k; ++j) {
                        const int cur = a.order[(size_t)b * a.G + a.step * a.k + j];
                        const int prev = a.d_prev[b * a.k + j];
                        f |= (cur == x);
                        if (a.use_prev) f |= (prev == x);
                        const int c = a.center_prev ? prev : cur;
                        if (a.window > 0 && c >= 0) f |= (x >= c - a.win_lo && x <= c + a.win_hi);
                    }
                    return f;
                };
                auto is_cand = [&](int x) -> bool { return x >= a.blk_lo && x < a.blk_hi && mk[x] != 0 && in_set(x); };
                cand = is_cand(p);
                act = in_set(p);
                // shifted logits (Appendix B): the row before a candidate produces its prediction
                if (a.shift && !act && p + 1 < a.L) act = is_cand(p + 1);
            }
            int tot_a, tot_c;
            const int ia = block_excl_scan(act, wave_tot, &tot_a);
            const int ic = block_excl_scan(cand, wave_tot, &tot_c);
            if (act) {
                a.row_pos[row_base + ia] = p;
                a.row_seq[row_base + ia] = b;
            }
            if (cand) {
                // with shifted logits position p - 1 is active and precedes p directly in the row order
                a.cand_row[cand_base + ic] = row_base + ia - (a.shift ? 1 : 0);
                a.cand_pos[cand_base + ic] = p;
            }
            row_base += tot_a;
            cand_base += tot_c;
        }
    }
    if (threadIdx.x == 0) {
        a.row_off[a.batch] = row_base;
        a.cand_off[a.batch] = cand_base;
        a.counts[0] = row_base;
        a.counts[1] = cand_base;
    }
}

// ------------------------------------------------------------------------------------------------
// h[r] = embed[token at (seq, pos)], a[r] = RMSNorm(h[r]) * gain; stamps the row's position.
// ------------------------------------------------------------------------------------------------
template <typename T, int VPT, int NT>
__global__ __launch_bounds__(NT) void embed_norm_kernel(const T *__restrict__ embed,
                                                         const int *__restrict__ tokens,
                                                         const int *__restrict__ row_pos,
                                                         const int *__restrict__ row_seq,
                                                         const int *__restrict__ counts,
                                                         const float *__restrict__ gain, float *__restrict__ h,
                                                         T *__restrict__ a, int *__restrict__ stamp, int L,
                                                         int d, float eps, int step) {
    __shared__ float red[16];
    const int r = blockIdx.x;
    if (r >= counts[0]) return;
    const int b = row_seq[r], p = row_pos[r];
    const int tok = tokens[(size_t)b * L + p];
    if (threadIdx.x == 0) stamp[(size_t)b * L + p] = step;
    const T *e = embed + (size_t)tok * d;
    float v[VPT], ss = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        int c = threadIdx.x + NT * i;
        v[i] = c < d ? El<T>::ld(e + c) : 0.f;
        ss += v[i] * v[i];
    }
    ss = block_sum(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        int c = threadIdx.x + NT * i;
        if (c < d) {
            h[(size_t)r * d + c] = v[i];
            El<T>::st(a + (size_t)r * d + c, v[i] * rs * gain[c]);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// h[r] += sum_s partial[s][r]; a[r] = RMSNorm(h[r]) * gain (the next projection's input).
// ------------------------------------------------------------------------------------------------
// four consecutive outputs as one store
__device__ __forceinline__ void store4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ __forceinline__ void store4(bf16_t *p, float4 v) {
    uint2 w;
    w.x = (uint32_t)f2bf(v.x) | ((uint32_t)f2bf(v.y) << 16);
    w.y = (uint32_t)f2bf(v.z) | ((uint32_t)f2bf(v.w) << 16);
    *reinterpret_cast<uint2 *>(p) = w;
}
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// one workgroup of NT threads per row, V4 float4 per lane: d must be a multiple of 4 and at most 4 * NT * V4
template <typename T, int V4, int NT>
__global__ __launch_bounds__(NT) void residual_norm_kernel(const float *__restrict__ part, int splits,
                                                            size_t split_stride,
                                                            const int *__restrict__ counts,
                                                            const float *__restrict__ gain,
                                                            float *__restrict__ h, T *__restrict__ a, int d,
                                                            float eps) {
    __shared__ float red[16];
    const int r = blockIdx.x;
    if (r >= counts[0]) return;
    float4 v[V4], g[V4];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < V4; ++i) {
        const int c = (threadIdx.x + NT * i) * 4;
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        g[i] = x;
        if (c < d) {
            const size_t at = (size_t)r * d + c;
            x = *reinterpret_cast<const float4 *>(h + at);
            g[i] = *reinterpret_cast<const float4 *>(gain + c);      // fetched with the row, not after the reduction
#pragma unroll 4
            for (int s = 0; s < splits; ++s) x = add4(x, *reinterpret_cast<const float4 *>(part + s * split_stride + at));
        }
        v[i] = x;
        ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
    }
    ss = block_sum(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int i = 0; i < V4; ++i) {
        const int c = (threadIdx.x + NT * i) * 4;
        if (c < d) {
            const size_t at = (size_t)r * d + c;
            *reinterpret_cast<float4 *>(h + at) = v[i];
            store4(a + at, make_float4(v[i].x * rs * g[i].x, v[i].y * rs * g[i].y, v[i].z * rs * g[i].z,
                                       v[i].w * rs * g[i].w));
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Rotary embedding of q and k with the row's true position (Appendix A: positional embeddings follow
// the token), q to its row buffer, k and v to the cache rows of that position (Algorithm 1 line 4,
// position-indexed instead of concatenated).
// qkv partials: [splits][rows][(Hq + 2 Hkv) * dh] fp32. rope: [L][dh/2] (cos, sin). dh % 8 == 0.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void rope_scatter_kernel(const float *__restrict__ part, int splits,
                                                           size_t split_stride,
                                                           const int *__restrict__ row_pos,
                                                           const int *__restrict__ row_seq,
                                                           const int *__restrict__ counts,
                                                           const float2 *__restrict__ rope, T *__restrict__ q,
                                                           T *__restrict__ Kc, T *__restrict__ Vc, int Hq,
                                                           int Hkv, int dh, int L) {
    const int r = blockIdx.x;
    if (r >= counts[0]) return;
    const int b = row_seq[r], p = row_pos[r];
    const int half = dh >> 1, q4 = half >> 2, slots = Hq + 2 * Hkv, n = slots * dh;
    const float *src = part + (size_t)r * n;
    // grid.y workgroups share a row: many small workgroups hide the load latency better than one long loop
    for (int e = blockIdx.y * 256 + threadIdx.x; e < slots * q4; e += 256 * gridDim.y) {
        const int hs = e / q4, i = (e % q4) * 4;
        float4 x1 = make_float4(0.f, 0.f, 0.f, 0.f), x2 = x1;
#pragma unroll 4
        for (int s = 0; s < splits; ++s) {
            x1 = add4(x1, *reinterpret_cast<const float4 *>(src + s * split_stride + hs * dh + i));
            x2 = add4(x2, *reinterpret_cast<const float4 *>(src + s * split_stride + hs * dh + i + half));
        }
        if (hs < Hq + Hkv) {
            const float4 c01 = *reinterpret_cast<const float4 *>(rope + (size_t)p * half + i);       // cos0 sin0 cos1 sin1
            const float4 c23 = *reinterpret_cast<const float4 *>(rope + (size_t)p * half + i + 2);
            const float4 y1 = make_float4(x1.x * c01.x - x2.x * c01.y, x1.y * c01.z - x2.y * c01.w,
                                          x1.z * c23.x - x2.z * c23.y, x1.w * c23.z - x2.w * c23.w);
            const float4 y2 = make_float4(x2.x * c01.x + x1.x * c01.y, x2.y * c01.z + x1.y * c01.w,
                                          x2.z * c23.x + x1.z * c23.y, x2.w * c23.z + x1.w * c23.w);
            x1 = y1;
            x2 = y2;
        }
        T *dst;
        if (hs < Hq) dst = q + ((size_t)r * Hq + hs) * dh;
        else if (hs < Hq + Hkv) dst = Kc + (((size_t)b * Hkv + (hs - Hq)) * L + p) * dh;
        else dst = Vc + (((size_t)b * Hkv + (hs - Hq - Hkv)) * L + p) * dh;
        store4(dst + i, x1);
        store4(dst + i + half, x2);
    }
}

// f[r][j] = silu(gate_j) * up_j with gate/up interleaved in the projection output; two outputs per lane.
__device__ __forceinline__ void store2(float *p, float a, float b) { *reinterpret_cast<float2 *>(p) = make_float2(a, b); }
__device__ __forceinline__ void store2(bf16_t *p, float a, float b) {
    *reinterpret_cast<uint32_t *>(p) = (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16);
}
template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const float *__restrict__ part, int splits,
                                                     size_t split_stride, const int *__restrict__ counts,
                                                     T *__restrict__ f, int F, int fast_exp) {
    const int r = blockIdx.y;
    if (r >= counts[0]) return;
    const int j = (blockIdx.x * 256 + threadIdx.x) * 2;
    if (j >= F) return;
    const float *src = part + (size_t)r * 2 * F + 2 * j;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);      // gate_j up_j gate_j+1 up_j+1
#pragma unroll 4
    for (int s = 0; s < splits; ++s) v = add4(v, *reinterpret_cast<const float4 *>(src + s * split_stride));
    const float s0 = v.x / (1.0f + (fast_exp ? __expf(-v.x) : expf(-v.x)));
    const float s1 = v.z / (1.0f + (fast_exp ? __expf(-v.z) : expf(-v.z)));
    store2(f + (size_t)r * F + j, s0 * v.y, s1 * v.w);
}

// dst[c] = src[cand_row[c]] (the rows that go through the vocabulary projection)
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_kernel(const T *__restrict__ src,
                                                          const int *__restrict__ cand_row,
                                                          const int *__restrict__ counts, T *__restrict__ dst,
                                                          int d) {
    const int c = blockIdx.x;
    if (c >= counts[1]) return;
    const T *s = src + (size_t)cand_row[c] * d;
    for (int i = threadIdx.x; i < d; i += 256) dst[(size_t)c * d + i] = s[i];
}

// out[m][n] = sum_s part[s][m][n]
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ part, int splits,
                                                              size_t split_stride, float *__restrict__ out,
                                                              size_t total) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float v = 0.f;
    for (int s = 0; s < splits; ++s) v += part[s * split_stride + i];
    out[i] = v;
}

// ------------------------------------------------------------------------------------------------
// Per candidate row: token = arg max of the logits with MASK excluded (lowest id on ties),
// confidence = its softmax probability (Sec. 3.1: keep the most confident predictions).
// ------------------------------------------------------------------------------------------------
// Two kernels: the vocabulary is cut into HEAD_SLICES ranges so that a handful of candidate rows still
// occupies the chip; every (row, range) block makes one pass keeping a running (max, sum of exp, arg max),
// the second kernel merges the ranges of a row.
__device__ __forceinline__ void head_merge(float &m, float &s, int &i, float om, float os, int oi) {
    if (om > m || (om == m && oi < i)) {
        s = s * expf(m - om) + os;       // m == -inf only with s == 0: exp(-inf) * 0 is never formed as inf * 0
        m = om;
        i = oi;
    } else if (om > -INFINITY) {
        s += os * expf(om - m);
    }
}

__global__ __launch_bounds__(256) void head_stats_partial_kernel(const float *__restrict__ logits,
                                                                 const int *__restrict__ counts, int V,
                                                                 int mask_id, HeadPartial *__restrict__ part) {
    __shared__ float sm[4], ss[4];
    __shared__ int si[4], sn[4];
    const int c = blockIdx.y, slice = blockIdx.x;
    if (c >= counts[1]) return;
    const int per = ((V + HEAD_SLICES - 1) / HEAD_SLICES + 3) & ~3;      // multiple of 4: aligned float4 loads
    const int v0 = slice * per, v1 = min(V, v0 + per);
    const float *row = logits + (size_t)c * V;
    float m = -INFINITY, sum = 0.f;
    int bi = 0x7fffffff;
    bool nan = false;
    auto take = [&](float x, int v) {
        if (v == mask_id) return;
        nan |= (x != x);
        if (x > m) {                     // ascending v per thread: the first maximum wins
            sum = sum * expf(m - x) + 1.f;
            m = x;
            bi = v;
        } else {
            sum += expf(x - m);
        }
    };
    const bool vec = ((size_t)c * V) % 4 == 0;          // row start 16-byte aligned
    if (vec) {
        for (int v = v0 + 4 * threadIdx.x; v < v1; v += 4 * 256) {
            if (v + 3 < v1) {
                const float4 x = *reinterpret_cast<const float4 *>(row + v);
                take(x.x, v); take(x.y, v + 1); take(x.z, v + 2); take(x.w, v + 3);
            } else {
                for (int u = v; u < v1; ++u) take(row[u], u);
            }
        }
    } else {
        for (int v = v0 + threadIdx.x; v < v1; v += 256) take(row[v], v);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        head_merge(m, sum, bi, __shfl_xor(m, o, 64), __shfl_xor(sum, o, 64), __shfl_xor(bi, o, 64));
    const int w = threadIdx.x >> 6;
    const bool any_nan = __any(nan);
    if ((threadIdx.x & 63) == 0) { sm[w] = m; ss[w] = sum; si[w] = bi; sn[w] = any_nan; }
    __syncthreads();
    if (threadIdx.x == 0) {
        int n = sn[0];
        for (int i = 1; i < 4; ++i) {
            head_merge(m, sum, bi, sm[i], ss[i], si[i]);
            n |= sn[i];
        }
        part[(size_t)c * HEAD_SLICES + slice] = HeadPartial{m, sum, bi, n};
    }
}

__global__ __launch_bounds__(256) void head_stats_final_kernel(const HeadPartial *__restrict__ part, int n_part,
                                                               const int *__restrict__ counts,
                                                               int *__restrict__ tok, float *__restrict__ conf,
                                                               int *__restrict__ status) {
    // one wavefront per candidate row; the merge keeps the lower token id on equal maxima in any order
    const int lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= counts[1]) return;
    float m = -INFINITY, sum = 0.f;
    int bi = 0x7fffffff, nan = 0;
    for (int s = lane; s < n_part; s += 64) {
        const HeadPartial p = part[(size_t)c * n_part + s];
        head_merge(m, sum, bi, p.max, p.sum, p.idx);
        nan |= p.nan;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        head_merge(m, sum, bi, __shfl_xor(m, o, 64), __shfl_xor(sum, o, 64), __shfl_xor(bi, o, 64));
    if (__any(nan) && lane == 0) atomicOr(status, STATUS_NAN);
    if (lane == 0) {
        tok[c] = bi;
        conf[c] = 1.0f / sum;
    }
}

// ------------------------------------------------------------------------------------------------
// Commit k positions per sequence: highest confidence first, ties to the lower position; or the
// forced / pre-ordered positions. Updates tokens, mask bitmap, the previous-commit list and the logs.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void commit_kernel(CommitArgs a) {
    __shared__ float sval[4];
    __shared__ int sidx[4];
    __shared__ int chosen;
    const int b = blockIdx.x;
    const int c0 = a.cand_off[b], c1 = a.cand_off[b + 1];
    for (int c = c0 + threadIdx.x; c < c1; c += 256) a.taken[c] = 0;
    __syncthreads();
    for (int j = 0; j < a.k; ++j) {
        int pick = -1;        // candidate index
        int want_pos = -1;
        if (a.forced_pos) want_pos = a.forced_pos[b * a.k + j];
        else if (a.order) want_pos = a.order[(size_t)b * a.G + a.step * a.k + j];
        if (want_pos >= 0) {
            if (threadIdx.x == 0) chosen = -1;
            __syncthreads();
            for (int c = c0 + threadIdx.x; c < c1; c += 256)
                if (a.cand_pos[c] == want_pos) chosen = c;
            __syncthreads();
            pick = chosen;
        } else {
            float best = -INFINITY;
            int bi = -1;
            for (int c = c0 + threadIdx.x; c < c1; c += 256) {
                float v = a.taken[c] ? -INFINITY : a.cand_conf[c];
                if (bi < 0 || v > best) { best = v; bi = c; }   // ascending c = ascending position
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                float ob = __shfl_xor(best, o, 64);
                int oi = __shfl_xor(bi, o, 64);
                if (oi >= 0 && (bi < 0 || ob > best || (ob == best && oi < bi))) { best = ob; bi = oi; }
            }
            __syncthreads();
            if ((threadIdx.x & 63) == 0) { sval[threadIdx.x >> 6] = best; sidx[threadIdx.x >> 6] = bi; }
            __syncthreads();
            best = sval[0]; bi = sidx[0];
            for (int i = 1; i < 4; ++i)
                if (sidx[i] >= 0 && (bi < 0 || sval[i] > best || (sval[i] == best && sidx[i] < bi))) {
                    best = sval[i]; bi = sidx[i];
                }
            pick = (bi >= 0 && !(best == -INFINITY)) ? bi : -1;
        }
        if (threadIdx.x == 0) {
            const size_t lo = ((size_t)a.step * a.batch + b) * a.k + j;
            if (pick < 0) {
                atomicOr(a.status, STATUS_BAD_COMMIT);
                a.d_prev[b * a.k + j] = -1;
                a.log_pos[lo] = -1; a.log_tok[lo] = -1; a.log_conf[lo] = 0.f;
            } else {
                const int p = a.cand_pos[pick];
                const int t = a.forced_tok ? a.forced_tok[b * a.k + j] : a.cand_tok[pick];
                a.tokens[(size_t)b * a.L + p] = t;
                a.masked[(size_t)b * a.L + p] = 0;
                a.taken[pick] = 1;
                a.d_prev[b * a.k + j] = p;
                a.log_pos[lo] = p; a.log_tok[lo] = t; a.log_conf[lo] = a.cand_conf[pick];
            }
        }
        __syncthreads();
    }
}

__global__ void init_state_kernel(int *tokens, uint8_t *masked, int *stamp, int *d_prev, int *status,
                                  int batch, int L, int P, int k, int mask_id) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (size_t)batch * L) {
        const int p = (int)(i % L);
        if (p >= P) tokens[i] = mask_id;
        masked[i] = p >= P;
        stamp[i] = -1;
    }
    if (i < (size_t)batch * k) d_prev[i] = -1;
    if (i == 0) *status = 0;
}

// Rotary angles of every (position, pair): the rotation follows the token's true position (Appendix A).
__global__ void rope_table_kernel(float2 *table, int L, int half, double theta) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)L * half) return;
    const int p = (int)(i / half), j = (int)(i % half);
    const double ang = (double)p * pow(theta, -(double)j / (double)half);
    table[i] = make_float2((float)cos(ang), (float)sin(ang));
}

__global__ void fill_i32_kernel(int *p, int v, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
__global__ void fill_u8_kernel(uint8_t *p, uint8_t v, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// k_cache[b][:, p, :] = k_new[r], v likewise (the scatter half of dkv_attn_update): 16-byte pieces, one per lane;
// a (row, head) is dh * sizeof(T) contiguous bytes on both sides (cpr pieces)
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint4 *__restrict__ k_new,
                                                           const uint4 *__restrict__ v_new,
                                                           const int *__restrict__ idx,
                                                           const int *__restrict__ off, uint4 *__restrict__ Kc,
                                                           uint4 *__restrict__ Vc, int batch, int Hkv, int L,
                                                           int cpr) {
    const int r = blockIdx.x;
    if (r >= off[batch]) return;
    int b = 0;
    while (r >= off[b + 1]) ++b;
    const int p = idx[r];
    for (int e = threadIdx.x; e < Hkv * cpr; e += 256) {
        const int h = e / cpr, i = e % cpr;
        const size_t dst = (((size_t)b * Hkv + h) * L + p) * cpr + i;
        Kc[dst] = k_new[(size_t)r * Hkv * cpr + e];
        Vc[dst] = v_new[(size_t)r * Hkv * cpr + e];
    }
}

// The cache operator of Appendix A (concat_reorder), as an alternative layout to measure against: the
// compact cache rows and the freshly computed rows of a (sequence, head) are concatenated and gathered into the
// order given by `take` (the next step's cached rows first). 16-byte chunks, one per thread.
__global__ __launch_bounds__(256) void concat_reorder_kernel(const uint4 *__restrict__ k_cached,
                                                             const uint4 *__restrict__ v_cached,
                                                             const uint4 *__restrict__ k_new,
                                                             const uint4 *__restrict__ v_new,
                                                             const int *__restrict__ take,
                                                             uint4 *__restrict__ k_out, uint4 *__restrict__ v_out,
                                                             int n_cached, int n_new, int cpr) {
    const int L = n_cached + n_new;
    const int bh = blockIdx.y, b = blockIdx.z;                 // head, sequence
    const int H = gridDim.y;
    const long c = (long)blockIdx.x * 256 + threadIdx.x;       // chunk of this (sequence, head)
    if (c >= (long)L * cpr) return;
    const int row = (int)(c / cpr), ch = (int)(c % cpr);
    const int src = take[(size_t)b * L + row];
    const size_t pair = (size_t)b * H + bh;
    const uint4 *ks, *vs;
    if (src < n_cached) {
        ks = k_cached + (pair * n_cached + src) * cpr + ch;
        vs = v_cached + (pair * n_cached + src) * cpr + ch;
    } else {
        ks = k_new + (pair * n_new + (src - n_cached)) * cpr + ch;
        vs = v_new + (pair * n_new + (src - n_cached)) * cpr + ch;
    }
    k_out[(pair * L + row) * cpr + ch] = *ks;
    v_out[(pair * L + row) * cpr + ch] = *vs;
}

template <typename T> int vpt_dispatch_embed(hipStream_t s, int rows, int d, const T *embed, const int *tokens,
                                             const int *row_pos, const int *row_seq, const int *counts,
                                             const float *gain, float *h, T *a, int *stamp, int L, float eps,
                                             int step) {
#define GO(V, NT)                                                                                          \
    hipLaunchKernelGGL((embed_norm_kernel<T, V, NT>), dim3(rows), dim3(NT), 0, s, embed, tokens, row_pos,  \
                       row_seq, counts, gain, h, a, stamp, L, d, eps, step)
    if (d <= 256) GO(1, 256);
    else if (d <= 1024) GO(1, 1024);
    else if (d <= 4096) GO(4, 1024);
    else if (d <= 8192) GO(8, 1024);
    else { dkv_set_error("d_model %d above 8192 is not supported", d); return DKV_E_UNSUPPORTED; }
#undef GO
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

template <typename T> int vpt_dispatch_resnorm(hipStream_t s, int rows, int d, const float *part, int splits,
                                               size_t stride, const int *counts, const float *gain, float *h,
                                               T *a, float eps) {
#define GO(V, NT)                                                                                          \
    hipLaunchKernelGGL((residual_norm_kernel<T, V, NT>), dim3(rows), dim3(NT), 0, s, part, splits, stride, \
                       counts, gain, h, a, d, eps)
    if (d % 4) { dkv_set_error("d_model %d must be a multiple of 4", d); return DKV_E_UNSUPPORTED; }
    // one float4 per lane per slice where the row is long enough: more wavefronts per row hide the load latency
    if (d <= 1024) GO(1, 256);
    else if (d <= 2048) GO(1, 512);
    else if (d <= 4096) GO(1, 1024);
    else if (d <= 8192) GO(2, 1024);
    else { dkv_set_error("d_model %d above 8192 is not supported", d); return DKV_E_UNSUPPORTED; }
#undef GO
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------- launchers

int dkv_launch_select(const SelectArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(select_active_kernel, dim3(1), dim3(1024), 0, s, a);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_embed_norm(int dtype, hipStream_t s, int rows, int d, const void *embed, const int *tokens,
                          const int *row_pos, const int *row_seq, const int *counts, const float *gain,
                          float *h, void *a, int *stamp, int L, float eps, int step) {
    if (rows <= 0) return DKV_OK;
    if (dtype == DKV_BF16)
        return vpt_dispatch_embed<bf16_t>(s, rows, d, (const bf16_t *)embed, tokens, row_pos, row_seq, counts,
                                          gain, h, (bf16_t *)a, stamp, L, eps, step);
    return vpt_dispatch_embed<float>(s, rows, d, (const float *)embed, tokens, row_pos, row_seq, counts, gain,
                                     h, (float *)a, stamp, L, eps, step);
}

int dkv_launch_residual_norm(int dtype, hipStream_t s, int rows, int d, const float *part, int splits,
                             size_t stride, const int *counts, const float *gain, float *h, void *a,
                             float eps) {
    if (rows <= 0) return DKV_OK;
    if (dtype == DKV_BF16)
        return vpt_dispatch_resnorm<bf16_t>(s, rows, d, part, splits, stride, counts, gain, h, (bf16_t *)a,
                                            eps);
    return vpt_dispatch_resnorm<float>(s, rows, d, part, splits, stride, counts, gain, h, (float *)a, eps);
}

int dkv_launch_rope_scatter(int dtype, hipStream_t s, int rows, const float *part, int splits, size_t stride,
                            const int *row_pos, const int *row_seq, const int *counts, const float *rope,
                            void *q, void *Kc, void *Vc, int Hq, int Hkv, int dh, int L) {
    if (rows <= 0) return DKV_OK;
    const int per_row = (Hq + 2 * Hkv) * (dh / 8);          // float4 pairs of a row
    int gy = ceil_div(per_row, 256);
    if (gy > 8) gy = 8;
    const dim3 grid(rows, gy);
    if (dtype == DKV_BF16)
        hipLaunchKernelGGL((rope_scatter_kernel<bf16_t>), grid, dim3(256), 0, s, part, splits, stride,
                           row_pos, row_seq, counts, (const float2 *)rope, (bf16_t *)q, (bf16_t *)Kc,
                           (bf16_t *)Vc, Hq, Hkv, dh, L);
    else
        hipLaunchKernelGGL((rope_scatter_kernel<float>), grid, dim3(256), 0, s, part, splits, stride,
                           row_pos, row_seq, counts, (const float2 *)rope, (float *)q, (float *)Kc,
                           (float *)Vc, Hq, Hkv, dh, L);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_swiglu(int dtype, hipStream_t s, int rows, const float *part, int splits, size_t stride,
                      const int *counts, void *f, int F) {
    if (rows <= 0) return DKV_OK;
    dim3 grid(ceil_div(F, 512), rows);
    if (dtype == DKV_BF16)
        hipLaunchKernelGGL((swiglu_kernel<bf16_t>), grid, dim3(256), 0, s, part, splits, stride, counts,
                           (bf16_t *)f, F, 1);
    else
        hipLaunchKernelGGL((swiglu_kernel<float>), grid, dim3(256), 0, s, part, splits, stride, counts,
                           (float *)f, F, 0);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_gather_rows(int dtype, hipStream_t s, int cands, const void *src, const int *cand_row,
                           const int *counts, void *dst, int d) {
    if (cands <= 0) return DKV_OK;
    if (dtype == DKV_BF16)
        hipLaunchKernelGGL((gather_rows_kernel<bf16_t>), dim3(cands), dim3(256), 0, s, (const bf16_t *)src,
                           cand_row, counts, (bf16_t *)dst, d);
    else
        hipLaunchKernelGGL((gather_rows_kernel<float>), dim3(cands), dim3(256), 0, s, (const float *)src,
                           cand_row, counts, (float *)dst, d);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_reduce_partials(hipStream_t s, const float *part, int splits, size_t stride, float *out,
                               size_t total) {
    if (total == 0) return DKV_OK;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, part,
                       splits, stride, out, total);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

size_t dkv_head_stats_scratch_bytes(int cands) { return (size_t)cands * HEAD_SLICES * sizeof(HeadPartial); }

int dkv_launch_head_stats(hipStream_t s, int cands, const float *logits, const int *counts, int V,
                          int mask_id, int *tok, float *conf, int *status, void *scratch) {
    if (cands <= 0) return DKV_OK;
    HeadPartial *part = static_cast<HeadPartial *>(scratch);
    hipLaunchKernelGGL(head_stats_partial_kernel, dim3(HEAD_SLICES, cands), dim3(256), 0, s, logits, counts, V,
                       mask_id, part);
    DKV_LAUNCH_CHECK();
    hipLaunchKernelGGL(head_stats_final_kernel, dim3((cands + 3) / 4), dim3(256), 0, s, part, HEAD_SLICES, counts, tok,
                       conf, status);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_head_merge(hipStream_t s, int cands, const void *head_part, int n_part, const int *counts, int *tok,
                          float *conf, int *status) {
    if (cands <= 0) return DKV_OK;
    hipLaunchKernelGGL(head_stats_final_kernel, dim3((cands + 3) / 4), dim3(256), 0, s,
                       static_cast<const HeadPartial *>(head_part), n_part, counts, tok, conf, status);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_commit(const CommitArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(commit_kernel, dim3(a.batch), dim3(256), 0, s, a);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_init_state(hipStream_t s, int *tokens, uint8_t *masked, int *stamp, int *d_prev, int *status,
                          int batch, int L, int P, int k, int mask_id) {
    size_t n = (size_t)batch * L;
    if ((size_t)batch * k > n) n = (size_t)batch * k;
    hipLaunchKernelGGL(init_state_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, tokens, masked,
                       stamp, d_prev, status, batch, L, P, k, mask_id);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_rope_table(hipStream_t s, float *table, int L, int dh, double theta) {
    const size_t n = (size_t)L * (dh / 2);
    if (!n) return DKV_OK;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<float2 *>(table), L, dh / 2, theta);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_fill_i32(hipStream_t s, int *p, int v, size_t n) {
    if (!n) return DKV_OK;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, v, n);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_fill_u8(hipStream_t s, uint8_t *p, uint8_t v, size_t n) {
    if (!n) return DKV_OK;
    hipLaunchKernelGGL(fill_u8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, v, n);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_concat_reorder(hipStream_t s, const void *k_cached, const void *v_cached, const void *k_new,
                              const void *v_new, const int *take, void *k_out, void *v_out, int batch, int heads,
                              int n_cached, int n_new, int row_bytes) {
    const int L = n_cached + n_new, cpr = row_bytes / 16;
    if (L <= 0 || batch <= 0) return DKV_OK;
    dim3 grid((unsigned)(((long)L * cpr + 255) / 256), heads, batch);
    hipLaunchKernelGGL(concat_reorder_kernel, grid, dim3(256), 0, s, (const uint4 *)k_cached, (const uint4 *)v_cached,
                       (const uint4 *)k_new, (const uint4 *)v_new, take, (uint4 *)k_out, (uint4 *)v_out, n_cached,
                       n_new, cpr);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

int dkv_launch_scatter_rows(int dtype, hipStream_t s, int rows, const void *k_new, const void *v_new,
                            const int *idx, const int *off, void *Kc, void *Vc, int batch, int Hkv, int L,
                            int dh) {
    if (rows <= 0) return DKV_OK;
    const int row_bytes = dh * (dtype == DKV_BF16 ? 2 : 4);
    if (row_bytes % 16) { dkv_set_error("a cache row of %d bytes is not a multiple of 16", row_bytes); return DKV_E_UNSUPPORTED; }
    hipLaunchKernelGGL(scatter_rows_kernel, dim3(rows), dim3(256), 0, s, (const uint4 *)k_new, (const uint4 *)v_new, idx, off,
                       (uint4 *)Kc, (uint4 *)Vc, batch, Hkv, L, row_bytes / 16);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}
