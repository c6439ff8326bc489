// Bidirectional attention of the active queries over the full-length, position-indexed K/V cache
// (Eq. 4: softmax(Q^{A_t} K^{I T} / sqrt(d)) V^I, no mask; query heads of one group share a K/V head).
//
// bf16 kernels (attn_ksplit.h, attn_shared.h): a "query row" is an (active row, query head of the group)
// pair, handled in tiles of 16. Keys stream in tiles through LDS (K rows and a transposed copy of the V
// rows), the next tile's global loads are in flight while the current tile is multiplied. Scores are formed
// transposed (keys x queries) so the probabilities come out of the MFMA already laid out as the
// operand of the second product and never leave registers; the output accumulates transposed
// (head_dim x queries) with a running max / sum per query (online softmax). The key-split kernel deals
// the key tiles to the wavefronts of a workgroup and merges their states in LDS; the shared kernel
// gives every wavefront its own query tiles over one shared K/V tile. When the keys are also sliced
// across workgroups every workgroup writes (max, sum, unnormalised output) and attn_merge combines them.
//
// generic kernel (fp32 mode and odd head sizes): one wavefront per (row, query head), lanes stride
// over the keys, fp32 FMA, exact expf.
#include <atomic>

#include "common.h"

namespace {

constexpr int KT = 32;                 // keys per tile

template <int DH> struct AttnSmem {
    static constexpr int K_STRIDE = DH * 2 + 16;        // bytes per K row (+16 spreads the 16-byte fragment reads)
    static constexpr int V_STRIDE = DH * 2 + 32;        // bytes per V row (+32 spreads the transposing reads)
    static constexpr int K_BYTES = KT * K_STRIDE;
    static constexpr int V_BYTES = KT * V_STRIDE;
    static constexpr int WAVE_BYTES = K_BYTES + V_BYTES;
};

typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((address_space(3))) bf16x4 *lds_bf16x4_ptr;

// MFMA operand V^T[dim 16 mt + (lane & 15)][8 keys] from V rows stored as they are in the cache (row = key).
// ds_read_b64_tr_b16 works on blocks of 16 lanes: lane j points at 4 consecutive 16-bit elements, and lane i
// receives element i % 4 of the pieces of lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12. With lane j pointing
// at dims [16 mt + 4 (j % 4), +4) of key j / 4, lane i gets dim 16 mt + i of four consecutive keys. Two reads
// give the 8 keys of the lane's K group in the order the probabilities come out of the score MFMA:
// keys key0 + 4 g + {0..3} and key0 + 16 + 4 g + {0..3}, g = lane / 16. `vrow0` = address of (key 4 g + j / 4,
// dim 4 (j % 4)) of the tile, precomputed per lane.
__device__ __forceinline__ bf16x8 vt_operand(const unsigned char *vrow0, int mt, int v_stride, int key0) {
    const unsigned char *a = vrow0 + key0 * v_stride + mt * 32;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(a));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(a + 16 * v_stride));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Reductions over the four lanes that hold one query (lane, lane ^ 16, lane ^ 32, lane ^ 48), every lane getting the
// result: gfx950's row swaps (v_permlane16_swap exchanges the odd 16-lane rows of one register with the even rows of
// another, v_permlane32_swap the upper half of one with the lower half of another; applied to two copies of x they
// leave "my value" and "my partner's value" side by side). Two vector instructions per stage instead of an LDS
// round trip (ds_bpermute) with its index arithmetic, on the path between the two products of every key tile.
__device__ __forceinline__ void swap_rows16(float x, float &u, float &v) {
    const unsigned a = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane16_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    u = __builtin_bit_cast(float, r0);
    v = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ void swap_rows32(float x, float &u, float &v) {
    const unsigned a = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    u = __builtin_bit_cast(float, r0);
    v = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float query_lanes_max(float x) {
    float u, v;
    swap_rows16(x, u, v);
    x = fmaxf(u, v);
    swap_rows32(x, u, v);
    return fmaxf(u, v);
}
__device__ __forceinline__ float query_lanes_sum(float x) {
    float u, v;
    swap_rows16(x, u, v);
    x = u + v;
    swap_rows32(x, u, v);
    return u + v;
}

// One online-softmax step of a lane over NT sub-tiles of 16 keys (Eq. 4's softmax, streamed): st[jt][i] is the raw
// score of key key_base + 16 jt + i against this lane's query. Updates the running max (log2 domain) and sum,
// rescales the output accumulators, and returns the probabilities as bf16 MFMA operands: operand hh covers
// sub-tiles 2hh and 2hh+1. The running sum is not formed here: the caller multiplies the same operands with a row of
// ones (row_sum_operand) into l_acc, so the matrix pipe adds up exactly the rounded probabilities that enter the
// second product and the vector units are spared sixteen additions per lane and tile; l_acc is only rescaled here.
template <int NT, int NACC>
__device__ __forceinline__ void softmax_step(f32x4 (&st)[NT], float &m_run, f32x4 &l_acc, f32x4 (&acc)[NACC],
                                             bf16x8 (&pb)[NT / 2], int key_base, int L, bool masked,
                                             float scale_log2e) {
    if (masked) {              // wave-uniform: only the last tile of a sequence has keys past the end
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (key_base + 16 * jt + i >= L) st[jt][i] = -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int i = 0; i < 4; ++i) mx = fmaxf(mx, st[jt][i]);
    mx = query_lanes_max(mx);
    const float m_new = fmaxf(m_run, mx * scale_log2e);
    // Rescale only when some query of the wavefront got a new maximum (rare after the first tiles): for the
    // others the factor would be exactly 1.
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_acc *= alpha;
#pragma unroll
        for (int mt = 0; mt < NACC; ++mt) acc[mt] *= alpha;
        m_run = m_new;
    }
#pragma unroll
    for (int hh = 0; hh < NT / 2; ++hh) {
        f32x8 p;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            p[e] = __builtin_amdgcn_exp2f(fmaf(st[2 * hh + (e >> 2)][e & 3], scale_log2e, -m_new));
        pb[hh] = __builtin_convertvector(p, bf16x8);
    }
}

// First operand of the product that sums the probabilities of a query: a 16 x 32 tile whose row 0 is all ones (the
// lanes with lane % 16 == 0 hold that row). mfma(row_sum_operand, pb, l_acc) adds the sum over the 32 keys of pb to
// element 0 of l_acc in the lanes below 16 (row 0, column = query); everything else in l_acc stays zero, so the sum
// over a query's four lanes (query_lanes_sum of element 0) is the running sum.
__device__ __forceinline__ bf16x8 row_sum_operand(int lane) {
    const __bf16 one = (lane & 15) == 0 ? (__bf16)1.0f : (__bf16)0.0f;
    return bf16x8{one, one, one, one, one, one, one, one};
}

// 16 bytes with the non-temporal hint (data that this launch reads once)
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_nt(const void *p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 16 bytes, plain
__device__ __forceinline__ uint4 load16(const void *p) {
    const u32x4_t v = *reinterpret_cast<const u32x4_t *>(p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Work-item order of the bf16 kernels. The `inner` workgroups of a (sequence, kv head) pair (query groups or blocks
// x key slices) read the same K/V rows, and the hardware sends workgroup i to XCD i mod 8, each with an L2 of its
// own: consecutive ids would have every XCD fetch the pair's K/V once more (measured: 4.2x the K/V bytes from
// memory with four query blocks per pair). So pair p lives on XCD p mod 8: its workgroups take the ids
// p mod 8 + 8 (inner (p / 8) + w), w < inner, which are dispatched within a few ids of each other. The grid is
// padded to a multiple of 8 pairs; returns false for the padding.
__device__ __forceinline__ bool attn_item(unsigned id, int pairs, int inner, int &pair, int &within) {
    const unsigned xcd = id & 7, slot = id >> 3;
    pair = (int)(slot / inner) * 8 + (int)xcd;
    within = (int)(slot % inner);
    return pair < pairs;
}
static inline unsigned attn_grid(long pairs, int inner) { return (unsigned)((pairs + 7) / 8 * 8 * inner); }

#include "attn_shared.h"
#include "attn_ksplit.h"

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
    p.shared_waves = 0;
    p.q_blocks = 0;
    p.ksplit_nq = 0;
    p.ksplit_waves = 0;
    p.q_groups = 0;
    int G = n_q_heads / n_kv_heads;
    p.q_tiles = ceil_div(max_rows_per_seq * G, 16);
    if (p.q_tiles < 1) p.q_tiles = 1;
    if (!p.use_mfma) {
        p.splits = 1;
        p.tiles_per_split = ceil_div(seq_len, KT);
        return p;
    }
    // Measured on MI355X over the shapes of the four workloads: the shared-tile kernel (about 450 TFLOP/s when
    // compute bound, against 200 for the key-split kernel, and K/V read from L2 once per 128 query rows) wins
    // as soon as its blocks of 8 query tiles make enough workgroups to occupy the chip without slicing the
    // keys, even when the last block of a head is mostly empty; below that the key-split kernel does.
    const int blocks8 = ceil_div(p.q_tiles, 8);
    const bool shared = head_dim == 128 && p.q_tiles >= 5 && (long)batch * n_kv_heads * blocks8 >= 192;
    int s = 1, n_tiles, min_tiles;
    if (shared) {
        // Blocks of 8 query tiles either way. With fewer than two workgroups per compute unit, 8 wavefronts
        // with one query tile each: a second wavefront per SIMD fills the waits of the first (softmax between
        // the two products, the tile barrier), which two co-resident workgroups do otherwise.
        const bool wide = (long)batch * n_kv_heads * blocks8 < 512;
        p.shared_nq = wide ? 1 : 2;
        p.shared_waves = wide ? 8 : 4;
        p.q_blocks = blocks8;
        n_tiles = ceil_div(seq_len, 64);
        min_tiles = 2;
    } else {
        p.ksplit_nq = p.q_tiles >= 2 ? 2 : 1;
        p.q_groups = ceil_div(p.q_tiles, p.ksplit_nq);
        n_tiles = ceil_div(seq_len, KT);
        const long items = (long)batch * n_kv_heads * p.q_groups;
        // 8 wavefronts per workgroup (one workgroup per compute unit) while that still gives every compute
        // unit at most one; beyond, 4 wavefronts so that two workgroups share a unit
        p.ksplit_waves = items <= 256 ? 8 : 4;
        if (items < 192) s = (int)((384 + items - 1) / items);
        min_tiles = 2 * p.ksplit_waves;                     // two tiles per wavefront
    }
    const int max_s = n_tiles / min_tiles > 0 ? n_tiles / min_tiles : 1;
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

int dkv_attn_can_fuse_update(const AttnPlan &plan, int max_rows_per_seq) {
    return plan.use_mfma && plan.ksplit_nq > 0 && max_rows_per_seq <= 64;
}

int dkv_launch_attention(int dtype, const void *q, void *k_cache, void *v_cache, const int *row_off, void *out,
                         int batch, int n_q_heads, int n_kv_heads, int seq_len, int head_dim, int rows_upper,
                         AttnPlan plan, void *partial, AttnFusedUpdate fuse, hipStream_t stream) {
    if (rows_upper <= 0) return DKV_OK;
    if (fuse.k_new && !plan.ksplit_nq) {
        dkv_set_error("the cache update can only be fused into the key-split attention kernel");
        return DKV_E_INVALID_ARG;
    }
    if (!plan.use_mfma) {
        if (dtype == DKV_BF16)
            return launch_generic<bf16_t>(q, k_cache, v_cache, row_off, out, batch, n_q_heads, n_kv_heads,
                                          seq_len, head_dim, rows_upper, stream);
        return launch_generic<float>(q, k_cache, v_cache, row_off, out, batch, n_q_heads, n_kv_heads,
                                     seq_len, head_dim, rows_upper, stream);
    }
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
    long pairs = (long)rows_upper * n_q_heads;
    if (plan.ksplit_nq) {
        const unsigned wgs = attn_grid((long)batch * n_kv_heads, plan.q_groups * plan.splits);
#define KSPLIT_F(D, NQ, NW, F)                                                                                 \
    do {                                                                                                       \
        static std::atomic<bool> lds_ok{false};    /* idempotent call: racing threads only repeat it */       \
        const size_t smem = NW * AttnSmem<D>::WAVE_BYTES;                                                      \
        if (!lds_ok.load(std::memory_order_acquire)) {                                                         \
            DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_ksplit<D, NQ, NW, F>),   \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));           \
            lds_ok.store(true, std::memory_order_release);                                                     \
        }                                                                                                      \
        hipLaunchKernelGGL((attn_bf16_ksplit<D, NQ, NW, F>), dim3(wgs), dim3(64 * NW), smem, stream,           \
                           (const bf16_t *)q, (bf16_t *)k_cache, (bf16_t *)v_cache, row_off, (bf16_t *)out,    \
                           (float *)partial, batch, n_q_heads, n_kv_heads, seq_len, plan.q_groups,             \
                           plan.splits, plan.tiles_per_split, rows_upper, scale_log2e,                         \
                           (const bf16_t *)fuse.k_new, (const bf16_t *)fuse.v_new, fuse.active_idx);           \
    } while (0)
#define KSPLIT(D, NQ, NW)                                                                                      \
    do {                                                                                                       \
        if (fuse.k_new) KSPLIT_F(D, NQ, NW, true);                                                             \
        else KSPLIT_F(D, NQ, NW, false);                                                                       \
    } while (0)
        if (head_dim == 128) {
            if (plan.ksplit_waves == 8) {
                if (plan.ksplit_nq == 2) KSPLIT(128, 2, 8);
                else KSPLIT(128, 1, 8);
            } else {
                if (plan.ksplit_nq == 2) KSPLIT(128, 2, 4);
                else KSPLIT(128, 1, 4);
            }
        } else {
            if (plan.ksplit_waves == 8) {
                if (plan.ksplit_nq == 2) KSPLIT(64, 2, 8);
                else KSPLIT(64, 1, 8);
            } else {
                if (plan.ksplit_nq == 2) KSPLIT(64, 2, 4);
                else KSPLIT(64, 1, 4);
            }
        }
#undef KSPLIT_F
#undef KSPLIT
        DKV_LAUNCH_CHECK();
        if (plan.splits > 1) {
            if (head_dim == 128)
                hipLaunchKernelGGL((attn_merge<128>), dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, stream,
                                   (const float *)partial, (bf16_t *)out, row_off, batch, n_q_heads, plan.splits,
                                   rows_upper);
            else
                hipLaunchKernelGGL((attn_merge<64>), dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, stream,
                                   (const float *)partial, (bf16_t *)out, row_off, batch, n_q_heads, plan.splits,
                                   rows_upper);
            DKV_LAUNCH_CHECK();
        }
    } else if (plan.shared_nq) {
        const size_t smem = 2 * 64 * ((128 * 2 + 16) + (128 * 2 + 32));   // two stages of 64 K rows and 64 V rows
        const unsigned wgs = attn_grid((long)batch * n_kv_heads, plan.q_blocks * plan.splits);
        static std::atomic<bool> lds_ok{false};
        if (!lds_ok.load(std::memory_order_acquire)) {
            DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_shared<2, 4, false>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_shared<2, 4, true>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_shared<1, 8, false>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_shared<1, 8, true>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            lds_ok.store(true, std::memory_order_release);
        }
#define SHARED(NQ_, NW_, ONCE_)                                                                                   \
    hipLaunchKernelGGL((attn_bf16_shared<NQ_, NW_, ONCE_>), dim3(wgs), dim3(64 * NW_), smem, stream, (const bf16_t *)q,  \
                       (const bf16_t *)k_cache, (const bf16_t *)v_cache, row_off, (bf16_t *)out, (float *)partial, \
                       batch, n_q_heads, n_kv_heads, seq_len, plan.q_blocks, plan.splits, plan.tiles_per_split,    \
                       rows_upper, scale_log2e)
        const bool once = plan.q_blocks == 1;       // nobody else reads the K/V rows of a workgroup
        if (plan.shared_waves == 8) {
            if (once) SHARED(1, 8, true);
            else SHARED(1, 8, false);
        } else {
            if (once) SHARED(2, 4, true);
            else SHARED(2, 4, false);
        }
#undef SHARED
        DKV_LAUNCH_CHECK();
        if (plan.splits > 1) {
            hipLaunchKernelGGL((attn_merge<128>), dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, stream,
                               (const float *)partial, (bf16_t *)out, row_off, batch, n_q_heads, plan.splits,
                               rows_upper);
            DKV_LAUNCH_CHECK();
        }
    }
    return DKV_OK;
}
