// Bidirectional attention of the active queries over the full-length, position-indexed K/V cache
// (Eq. 4: softmax(Q^{A_t} K^{I T} / sqrt(d)) V^I, no mask; query heads of one group share a K/V head).
//
// bf16 kernel: one wavefront owns one work item = (sequence, kv head, 16 query rows, key slice), where
// a "query row" is an (active row, query head of the group) pair. It streams its key slice in tiles
// of 32 keys: K rows and a transposed copy of the V rows go through a wave-private LDS region, the
// next tile's global loads are in flight while the current tile is multiplied. Scores are formed
// transposed (keys x queries) so the probabilities come out of the MFMA already laid out as the
// operand of the second product and never leave registers; the output accumulates transposed
// (head_dim x queries) with a running max / sum per query (online softmax). With several key
// slices every item writes (max, sum, unnormalised output) and a second kernel merges them.
//
// generic kernel (fp32 mode and odd head sizes): one wavefront per (row, query head), lanes stride
// over the keys, fp32 FMA, exact expf.
#include "common.h"

namespace {

constexpr int KT = 32;                 // keys per tile

template <int DH> struct AttnSmem {
    static constexpr int K_STRIDE = DH * 2 + 16;        // bytes per key row (+16 spreads banks)
    static constexpr int VT_STRIDE = KT * 2 + 8;        // bytes per head-dim row of V^T
    static constexpr int K_BYTES = KT * K_STRIDE;
    static constexpr int VT_BYTES = DH * VT_STRIDE;
    static constexpr int WAVE_BYTES = K_BYTES + VT_BYTES;
};

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// One online-softmax step of a lane over NT sub-tiles of 16 keys (Eq. 4's softmax, streamed): st[jt][i] is the raw
// score of key key_base + 16 jt + i against this lane's query. Updates the running max (log2 domain) and sum,
// rescales the output accumulators, and returns the probabilities as bf16 MFMA operands: operand hh covers
// sub-tiles 2hh and 2hh+1. The sum uses the unrounded probabilities.
template <int NT, int NACC>
__device__ __forceinline__ void softmax_step(f32x4 (&st)[NT], float &m_run, float &l_run, f32x4 (&acc)[NACC],
                                             bf16x8 (&pb)[NT / 2], int key_base, int L, bool masked,
                                             float scale_log2e) {
    float mx = -INFINITY;
#pragma unroll
    for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (masked && key_base + 16 * jt + i >= L) st[jt][i] = -INFINITY;
            mx = fmaxf(mx, st[jt][i]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * scale_log2e);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int hh = 0; hh < NT / 2; ++hh) {
        f32x8 p;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(st[2 * hh + (e >> 2)][e & 3], scale_log2e, -m_new));
            psum += p[e];
        }
        pb[hh] = __builtin_convertvector(p, bf16x8);
    }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int mt = 0; mt < NACC; ++mt) acc[mt] *= alpha;
}

template <int DH>
__global__ __launch_bounds__(256) void attn_bf16_mfma(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ Kc, const bf16_t *__restrict__ Vc,
    const int *__restrict__ row_off, bf16_t *__restrict__ out, float *__restrict__ part, int batch,
    int Hq, int Hkv, int L, int q_tiles, int splits, int tiles_per_split, int rows_cap,
    float scale_log2e) {
    using SM = AttnSmem<DH>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned char *ksm = smem_raw + wave * SM::WAVE_BYTES;
    unsigned char *vsm = ksm + SM::K_BYTES;

    const int G = Hq / Hkv;
    long item = (long)blockIdx.x * 4 + wave;
    const long n_items = (long)batch * Hkv * q_tiles * splits;
    if (item >= n_items) return;
    const int split = (int)(item % splits); item /= splits;
    const int qt = (int)(item % q_tiles);   item /= q_tiles;
    const int kvh = (int)(item % Hkv);
    const int b = (int)(item / Hkv);

    const int r0 = row_off[b], nrows = row_off[b + 1] - r0;
    const int nq = nrows * G;                    // query rows of this (sequence, kv head)
    const int m0 = qt * 16;
    if (m0 >= nq) return;

    const int qi = lane & 15, g = lane >> 4;
    // my query column: (row, head)
    const int mq = m0 + qi;
    // rows beyond the host's bound have no slot in the output or partial buffers
    const bool q_ok = mq < nq && r0 + mq / G < rows_cap;
    const int q_row = q_ok ? r0 + mq / G : 0, q_head = kvh * G + (q_ok ? mq % G : 0);

    bf16x8 qf[DH / 32];
    {
        const bf16_t *qp = Q + ((size_t)q_row * Hq + q_head) * DH + 8 * g;
#pragma unroll
        for (int ks = 0; ks < DH / 32; ++ks) {
            uint4 v = q_ok ? *reinterpret_cast<const uint4 *>(qp + 32 * ks) : make_uint4(0, 0, 0, 0);
            qf[ks] = *reinterpret_cast<bf16x8 *>(&v);
        }
    }

    const bf16_t *Kb = Kc + ((size_t)b * Hkv + kvh) * (size_t)L * DH;
    const bf16_t *Vb = Vc + ((size_t)b * Hkv + kvh) * (size_t)L * DH;
    const int n_tiles = (L + KT - 1) / KT;
    const int t0 = split * tiles_per_split, t1 = min(n_tiles, t0 + tiles_per_split);

    // global -> register staging of one tile
    constexpr int KCH = KT * DH / 8 / 64;        // 16-byte K chunks per lane
    constexpr int VTASK = (KT / 4) * (DH / 8) / 64;   // (4 keys x 8 dims) transposition tasks per lane
    uint4 kreg[KCH], vreg[VTASK][4];
    auto load_tile = [&](int t) {
        const int key0 = t * KT;
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            int c = lane + 64 * i, key = c / (DH / 8), ch = c % (DH / 8);
            int gk = key0 + key;
            kreg[i] = gk < L ? *reinterpret_cast<const uint4 *>(Kb + (size_t)gk * DH + ch * 8)
                             : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < VTASK; ++i) {
            int task = lane + 64 * i, dc = task % (DH / 8), kg = task / (DH / 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int gk = key0 + 4 * kg + j;
                vreg[i][j] = gk < L ? *reinterpret_cast<const uint4 *>(Vb + (size_t)gk * DH + dc * 8)
                                    : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            int c = lane + 64 * i, key = c / (DH / 8), ch = c % (DH / 8);
            *reinterpret_cast<uint4 *>(ksm + key * SM::K_STRIDE + ch * 16) = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < VTASK; ++i) {
            int task = lane + 64 * i, dc = task % (DH / 8), kg = task / (DH / 8);
            const uint32_t *v0 = reinterpret_cast<const uint32_t *>(&vreg[i][0]);
            const uint32_t *v1 = reinterpret_cast<const uint32_t *>(&vreg[i][1]);
            const uint32_t *v2 = reinterpret_cast<const uint32_t *>(&vreg[i][2]);
            const uint32_t *v3 = reinterpret_cast<const uint32_t *>(&vreg[i][3]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {     // word e holds dims 2e (low half) and 2e+1 (high half)
                uint2 lo = make_uint2(pack_lo(v0[e], v1[e]), pack_lo(v2[e], v3[e]));
                uint2 hi = make_uint2(pack_hi(v0[e], v1[e]), pack_hi(v2[e], v3[e]));
                int d = dc * 8 + 2 * e;
                *reinterpret_cast<uint2 *>(vsm + d * SM::VT_STRIDE + kg * 8) = lo;
                *reinterpret_cast<uint2 *>(vsm + (d + 1) * SM::VT_STRIDE + kg * 8) = hi;
            }
        }
    };

    float m_run = -INFINITY, l_run = 0.f;
    f32x4 acc[DH / 16];
#pragma unroll
    for (int i = 0; i < DH / 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (t0 < t1) load_tile(t0);
    for (int t = t0; t < t1; ++t) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        store_tile();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (t + 1 < t1) load_tile(t + 1);

        // S^T[key][query] for the two 16-key halves of the tile
        f32x4 st[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            st[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            const unsigned char *krow = ksm + (16 * j + qi) * SM::K_STRIDE + g * 16;
#pragma unroll
            for (int ks = 0; ks < DH / 32; ++ks) {
                bf16x8 kf = *reinterpret_cast<const bf16x8 *>(krow + ks * 64);
                st[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[ks], st[j], 0, 0, 0);
            }
        }
        // st[j][i] belongs to key 16j + 4g + i and query qi
        bf16x8 pbv[1];
        softmax_step<2, DH / 16>(st, m_run, l_run, acc, pbv, t * KT + 4 * g, L, (t + 1) * KT > L, scale_log2e);
        const bf16x8 pb = pbv[0];
#pragma unroll
        for (int mt = 0; mt < DH / 16; ++mt) {
            const unsigned char *vrow = vsm + (16 * mt + qi) * SM::VT_STRIDE;
            uint2 a0 = *reinterpret_cast<const uint2 *>(vrow + g * 8);          // keys 4g..4g+3
            uint2 a1 = *reinterpret_cast<const uint2 *>(vrow + 32 + g * 8);     // keys 16+4g..
            uint4 av = make_uint4(a0.x, a0.y, a1.x, a1.y);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&av), pb, acc[mt],
                                                               0, 0, 0);
        }
    }

    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (!q_ok) return;
    if (splits == 1) {
        const float inv = 1.f / l_run;
        bf16_t *op = out + ((size_t)q_row * Hq + q_head) * DH;
#pragma unroll
        for (int mt = 0; mt < DH / 16; ++mt) {
            uint2 w;
            w.x = (uint32_t)f2bf(acc[mt][0] * inv) | ((uint32_t)f2bf(acc[mt][1] * inv) << 16);
            w.y = (uint32_t)f2bf(acc[mt][2] * inv) | ((uint32_t)f2bf(acc[mt][3] * inv) << 16);
            *reinterpret_cast<uint2 *>(op + 16 * mt + 4 * g) = w;
        }
    } else {
        // partial record per (query row-head, split): [m, l, pad, pad, o[DH]]
        float *rec = part + (((size_t)q_row * Hq + q_head) * splits + split) * (DH + 4);
        if (g == 0) {
            rec[0] = m_run;
            rec[1] = l_run;
        }
#pragma unroll
        for (int mt = 0; mt < DH / 16; ++mt)
            *reinterpret_cast<f32x4 *>(rec + 4 + 16 * mt + 4 * g) = acc[mt];
    }
}

#include "attn_shared.h"

// Merge the key slices of one (row, head): one wavefront per pair.
template <int DH>
__global__ __launch_bounds__(256) void attn_merge(const float *__restrict__ part, bf16_t *__restrict__ out,
                                                  const int *__restrict__ row_off, int batch, int Hq,
                                                  int splits, int rows_cap) {
    const int lane = threadIdx.x & 63;
    const long pair = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long n_pairs = (long)min(row_off[batch], rows_cap) * Hq;
    if (pair >= n_pairs) return;
    const float *rec = part + (size_t)pair * splits * (DH + 4);
    float M = -INFINITY;
    for (int s = 0; s < splits; ++s) M = fmaxf(M, rec[(size_t)s * (DH + 4)]);
    float lsum = 0.f;
    float o[DH / 64 > 0 ? DH / 64 : 1] = {};
    for (int s = 0; s < splits; ++s) {
        const float *r = rec + (size_t)s * (DH + 4);
        float w = exp2f(r[0] - M);
        lsum += w * r[1];
#pragma unroll
        for (int i = 0; i < (DH / 64 > 0 ? DH / 64 : 1); ++i) {
            int d = lane + 64 * i;
            if (d < DH) o[i] += w * r[4 + d];
        }
    }
    const float inv = 1.f / lsum;
#pragma unroll
    for (int i = 0; i < (DH / 64 > 0 ? DH / 64 : 1); ++i) {
        int d = lane + 64 * i;
        if (d < DH) out[(size_t)pair * DH + d] = f2bf(o[i] * inv);
    }
}

// Generic kernel: one wavefront per (row, head).
template <typename T, int DH>
__global__ __launch_bounds__(256) void attn_generic(const T *__restrict__ Q, const T *__restrict__ Kc,
                                                    const T *__restrict__ Vc,
                                                    const int *__restrict__ row_off, T *__restrict__ out,
                                                    int batch, int Hq, int Hkv, int L, int rows_cap,
                                                    float scale) {
    const int lane = threadIdx.x & 63;
    const long pair = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int total_rows = min(row_off[batch], rows_cap);
    if (pair >= (long)total_rows * Hq) return;
    const int row = (int)(pair / Hq), h = (int)(pair % Hq);
    int b = 0;
    while (row >= row_off[b + 1]) ++b;
    const int kvh = h / (Hq / Hkv);
    const T *qp = Q + (size_t)pair * DH;
    const T *Kb = Kc + ((size_t)b * Hkv + kvh) * (size_t)L * DH;
    const T *Vb = Vc + ((size_t)b * Hkv + kvh) * (size_t)L * DH;
    float q[DH], o[DH];
#pragma unroll
    for (int d = 0; d < DH; ++d) {
        q[d] = El<T>::ld(qp + d);
        o[d] = 0.f;
    }
    float m = -INFINITY, l = 0.f;
    for (int key = lane; key < L; key += 64) {
        const T *kp = Kb + (size_t)key * DH;
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < DH; ++d) s = fmaf(q[d], El<T>::ld(kp + d), s);
        s *= scale;
        float mn = fmaxf(m, s);
        float a = expf(m - mn), p = expf(s - mn);
        l = l * a + p;
        const T *vp = Vb + (size_t)key * DH;
#pragma unroll
        for (int d = 0; d < DH; ++d) o[d] = fmaf(p, El<T>::ld(vp + d), o[d] * a);
        m = mn;
    }
    const float Mx = wave_max(m);
    const float w = (m == -INFINITY) ? 0.f : expf(m - Mx);
    const float lt = wave_sum(l * w);
    const float inv = 1.f / lt;
#pragma unroll
    for (int d = 0; d < DH; ++d) {
        float v = wave_sum(o[d] * w);
        if (lane == (d & 63)) El<T>::st(out + (size_t)pair * DH + d, v * inv);
    }
}

template <typename T>
int launch_generic(const void *q, const void *k, const void *v, const int *row_off, void *out, int batch,
                   int Hq, int Hkv, int L, int dh, int rows_upper, hipStream_t s) {
    long pairs = (long)rows_upper * Hq;
    dim3 grid((unsigned)((pairs + 3) / 4));
    float scale = 1.0f / sqrtf((float)dh);
#define GEN(D)                                                                                        \
    hipLaunchKernelGGL((attn_generic<T, D>), grid, dim3(256), 0, s, (const T *)q, (const T *)k,       \
                       (const T *)v, row_off, (T *)out, batch, Hq, Hkv, L, rows_upper, scale)
    if (dh == 32) GEN(32);
    else if (dh == 64) GEN(64);
    else if (dh == 128) GEN(128);
    else {
        dkv_set_error("head_dim %d not supported (32, 64, 128)", dh);
        return DKV_E_UNSUPPORTED;
    }
#undef GEN
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

}  // namespace

AttnPlan dkv_attn_plan(int dtype, int batch, int n_q_heads, int n_kv_heads, int seq_len, int head_dim,
                       int max_rows_per_seq) {
    AttnPlan p;
    p.use_mfma = (dtype == DKV_BF16 && (head_dim == 64 || head_dim == 128)) ? 1 : 0;
    p.shared_nq = 0;
    p.q_blocks = 0;
    int G = n_q_heads / n_kv_heads;
    p.q_tiles = ceil_div(max_rows_per_seq * G, 16);
    if (p.q_tiles < 1) p.q_tiles = 1;
    int s = 1, n_tiles;
    if (p.use_mfma && head_dim == 128 && p.q_tiles >= 4) {
        // enough query rows to give every wavefront of a workgroup its own tile(s)
        p.shared_nq = p.q_tiles >= 8 ? 2 : 1;
        p.q_blocks = ceil_div(p.q_tiles, 4 * p.shared_nq);
        n_tiles = ceil_div(seq_len, 64);
        long items = (long)batch * n_kv_heads * p.q_blocks;
        if (items < 512) s = (int)((512 + items - 1) / items);
    } else {
        n_tiles = ceil_div(seq_len, KT);
        long items = (long)batch * n_kv_heads * p.q_tiles;
        if (p.use_mfma && items < 2048) s = (int)((2048 + items - 1) / items);
    }
    int max_s = n_tiles / 2 > 0 ? n_tiles / 2 : 1;      // at least two tiles per slice
    if (s > max_s) s = max_s;
    p.tiles_per_split = ceil_div(n_tiles, s);
    p.splits = ceil_div(n_tiles, p.tiles_per_split);
    return p;
}

size_t dkv_attn_partial_bytes(const AttnPlan &p, int batch, int n_q_heads, int n_kv_heads, int head_dim) {
    if (!p.use_mfma || p.splits == 1) return 0;
    int G = n_q_heads / n_kv_heads;
    // rows per sequence are at most q_tiles*16/G (rounded up); records are indexed by (row, head, split)
    size_t rows = (size_t)batch * (size_t)ceil_div(p.q_tiles * 16, G);
    return rows * n_q_heads * p.splits * (size_t)(head_dim + 4) * sizeof(float);
}

int dkv_launch_attention(int dtype, const void *q, const void *k_cache, const void *v_cache,
                         const int *row_off, void *out, int batch, int n_q_heads, int n_kv_heads,
                         int seq_len, int head_dim, int rows_upper, AttnPlan plan, void *partial,
                         hipStream_t stream) {
    if (rows_upper <= 0) return DKV_OK;
    if (!plan.use_mfma) {
        if (dtype == DKV_BF16)
            return launch_generic<bf16_t>(q, k_cache, v_cache, row_off, out, batch, n_q_heads, n_kv_heads,
                                          seq_len, head_dim, rows_upper, stream);
        return launch_generic<float>(q, k_cache, v_cache, row_off, out, batch, n_q_heads, n_kv_heads,
                                     seq_len, head_dim, rows_upper, stream);
    }
    long items = (long)batch * n_kv_heads * plan.q_tiles * plan.splits;
    dim3 grid((unsigned)((items + 3) / 4));
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
    long pairs = (long)rows_upper * n_q_heads;
    if (plan.shared_nq) {
        const size_t smem = 2 * (64 * (128 * 2 + 16) + 128 * (64 * 2 + 8));
        const unsigned wgs = (unsigned)((long)batch * n_kv_heads * plan.q_blocks * plan.splits);
        static bool lds_ok1 = false, lds_ok2 = false;
        if (plan.shared_nq == 1) {
            if (!lds_ok1) {
                DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_shared<1>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
                lds_ok1 = true;
            }
            hipLaunchKernelGGL((attn_bf16_shared<1>), dim3(wgs), dim3(256), smem, stream, (const bf16_t *)q,
                               (const bf16_t *)k_cache, (const bf16_t *)v_cache, row_off, (bf16_t *)out,
                               (float *)partial, batch, n_q_heads, n_kv_heads, seq_len, plan.q_blocks, plan.splits,
                               plan.tiles_per_split, rows_upper, scale_log2e);
        } else {
            if (!lds_ok2) {
                DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_shared<2>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
                lds_ok2 = true;
            }
            hipLaunchKernelGGL((attn_bf16_shared<2>), dim3(wgs), dim3(256), smem, stream, (const bf16_t *)q,
                               (const bf16_t *)k_cache, (const bf16_t *)v_cache, row_off, (bf16_t *)out,
                               (float *)partial, batch, n_q_heads, n_kv_heads, seq_len, plan.q_blocks, plan.splits,
                               plan.tiles_per_split, rows_upper, scale_log2e);
        }
        DKV_LAUNCH_CHECK();
        if (plan.splits > 1) {
            hipLaunchKernelGGL((attn_merge<128>), dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, stream,
                               (const float *)partial, (bf16_t *)out, row_off, batch, n_q_heads, plan.splits,
                               rows_upper);
            DKV_LAUNCH_CHECK();
        }
    } else if (head_dim == 128) {
        size_t smem = 4 * AttnSmem<128>::WAVE_BYTES;
        static bool lds_ok = false;
        if (!lds_ok) {
            DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_mfma<128>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            lds_ok = true;
        }
        hipLaunchKernelGGL((attn_bf16_mfma<128>), grid, dim3(256), smem, stream, (const bf16_t *)q,
                           (const bf16_t *)k_cache, (const bf16_t *)v_cache, row_off, (bf16_t *)out,
                           (float *)partial, batch, n_q_heads, n_kv_heads, seq_len, plan.q_tiles,
                           plan.splits, plan.tiles_per_split, rows_upper, scale_log2e);
        DKV_LAUNCH_CHECK();
        if (plan.splits > 1) {
            hipLaunchKernelGGL((attn_merge<128>), dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, stream,
                               (const float *)partial, (bf16_t *)out, row_off, batch, n_q_heads,
                               plan.splits, rows_upper);
            DKV_LAUNCH_CHECK();
        }
    } else {
        size_t smem = 4 * AttnSmem<64>::WAVE_BYTES;
        static bool lds_ok = false;
        if (!lds_ok) {
            DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_mfma<64>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            lds_ok = true;
        }
        hipLaunchKernelGGL((attn_bf16_mfma<64>), grid, dim3(256), smem, stream, (const bf16_t *)q,
                           (const bf16_t *)k_cache, (const bf16_t *)v_cache, row_off, (bf16_t *)out,
                           (float *)partial, batch, n_q_heads, n_kv_heads, seq_len, plan.q_tiles,
                           plan.splits, plan.tiles_per_split, rows_upper, scale_log2e);
        DKV_LAUNCH_CHECK();
        if (plan.splits > 1) {
            hipLaunchKernelGGL((attn_merge<64>), dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, stream,
                               (const float *)partial, (bf16_t *)out, row_off, batch, n_q_heads,
                               plan.splits, rows_upper);
            DKV_LAUNCH_CHECK();
        }
    }
    return DKV_OK;
}
