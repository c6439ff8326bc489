// Shared device/host helpers of the dKV-Cache HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/dkv.h"

typedef uint16_t bf16_t;   // raw bfloat16 bits

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) float f32x8;

#define DKV_WAVE 64

void dkv_set_error(const char *fmt, ...);

#define DKV_HIP_TRY(expr)                                                                  \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess) {                                                            \
            dkv_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                          __LINE__);                                                       \
            return DKV_E_HIP;                                                              \
        }                                                                                  \
    } while (0)

#define DKV_LAUNCH_CHECK()  DKV_HIP_TRY(hipGetLastError())

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest even (the hardware conversion); NaN stays NaN
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

template <typename T> struct El;
template <> struct El<float> {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
};
template <> struct El<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t *p) { return bf2f(*p); }
    static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f2bf(v); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Block-wide sum for blocks of up to 1024 threads (a multiple of 64); `red` holds >= 16 floats.
__device__ __forceinline__ float block_sum(float v, float *red) {
    v = wave_sum(v);
    int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += red[i];
    return t;
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- internal launchers (host side) --------------------------------------------------------

// Plan of one projection: tile shape and split of the K dimension.
enum { GEMM_DMA_32x128 = 0, GEMM_DMA_64x128, GEMM_DMA_128x128, GEMM_DMA_128x256, GEMM_DMA_256x256,
       GEMM_DMA_128x96, GEMM_DMA_128x192, GEMM_DMA_256x192, GEMM_DMA_192x256, GEMM_REG_64x128, GEMM_SIMT, GEMM_KINDS };
enum { GEMM_DMA_LAST = GEMM_DMA_192x256 };      // the gemm_dma tile kernels are the kinds 0 .. GEMM_DMA_LAST
enum { GEMM_FLAG_STAGGER = 1, GEMM_FLAG_XCD_GROUP = 2, GEMM_FLAG_SWIGLU = 4, GEMM_FLAG_STREAM_W = 8 };
struct GemmPlan {
    int kind;      // GEMM_* kernel and tile shape
    int split_k;   // number of partial slots: slice or part s writes partial[s]
    int frac_units; // 0, or K tiles per workgroup when workgroups take 3/4 of a tile's K range each
    int flags;     // GEMM_FLAG_* launch options of the gemm_dma kinds
};
GemmPlan dkv_gemm_plan(int dtype, int m_upper, int n, int k);
int dkv_gemm_plan_valid(int dtype, int k, GemmPlan p);

// Per (candidate row, vocabulary range): running maximum of the logits, sum of exp(x - max) over the range,
// index of the maximum (lowest on ties), and whether a NaN was seen.
struct HeadPartial {
    float max, sum;
    int idx, nan;
};

// What a projection launch (gemm_dma kinds) does with its finished tile. Only epilogues that do not have to load
// anything are fused: measured on MI355X, an epilogue that reads (residual rows, rotary angles, parked K slices) runs
// at the tail of a workgroup that has its compute unit to itself, nothing hides the latency of its loads, and it costs
// as much as, or more than, the row kernel it would replace.
enum {
    EPI_STORE = 0,   // partial[slice][m][n] = product of the K slice (fp32)
    EPI_SWIGLU,      // out[m][n/2] = silu(gate) * up (bf16); W rows interleave gate_j, up_j; one K slice
    EPI_HEAD         // vocabulary head: per row and column tile (max, sum exp, arg max) with MASK excluded; one K slice
};
struct GemmEpilogue {
    int kind = EPI_STORE;
    void *out = nullptr;              // EPI_SWIGLU: bf16 [m][N/2]; EPI_HEAD: fp32 logits [m][N] or null (not written)
    HeadPartial *head_part = nullptr; // EPI_HEAD: [m][head_tiles]
    int head_tiles = 0, mask_id = -1;
    int *status = nullptr;            // EPI_HEAD: STATUS_NAN is raised here
};
// Column tiles of a plan's kernel for N columns (the second dimension of head_part).
int dkv_gemm_tiles_n(const GemmPlan &plan, int n);
// The vocabulary projection with the softmax statistics in its epilogue (gemm_dma kinds, one K slice).
bool dkv_gemm_can_fuse_head(int dtype, int k, const GemmPlan &plan);
int dkv_launch_gemm_head(const void *A, const void *W, int m_upper, const int *m_dev, int n, int k, GemmPlan plan,
                         const GemmEpilogue &ep, hipStream_t stream);

// one translation unit per epilogue holds the tile kernels instantiated with it
#define DKV_DECLARE_DISPATCH(name)                                                                                   \
    int dkv_dispatch_dma_##name(const void *A, const void *W, float *partial, int m_upper, int m_cap, const int *m_dev, \
                                int n, int k, const GemmPlan &plan, const GemmEpilogue &ep, hipStream_t stream);
DKV_DECLARE_DISPATCH(store)
DKV_DECLARE_DISPATCH(swiglu)
DKV_DECLARE_DISPATCH(head)
#undef DKV_DECLARE_DISPATCH

// partial[s][m][n] (fp32, stride m_cap rows per slice) = A[m, k-slice] * W[n, k-slice]^T.
// Rows >= *m_dev (when m_dev != nullptr) are neither read nor written.
// With GEMM_FLAG_SWIGLU in plan.flags (gemm_dma kinds, one K slice, W rows interleaved gate_j, up_j): `partial` is
// instead a bf16 [m][n/2] array that receives silu(gate_j) * up_j, and no fp32 product is written.
bool dkv_gemm_can_fuse_swiglu(int dtype, int n, int k, const GemmPlan &p);
int dkv_launch_gemm(int dtype, const void *A, const void *W, float *partial, int m_upper, int m_cap,
                    const int *m_dev, int n, int k, GemmPlan plan, hipStream_t stream);

struct AttnPlan {
    int use_mfma;     // 1: bf16 MFMA kernel, 0: generic kernel
    int q_tiles;      // 16-row query tiles per (sequence, kv head), upper bound
    int splits;       // slices of the key range
    int tiles_per_split;   // in tiles of 32 keys (wave-private kernel) or 64 keys (shared kernel)
    int shared_nq;    // 0: one wavefront per item; 1 or 2: workgroup-shared K/V tiles, query tiles per wavefront
    int shared_waves; // shared kernel: wavefronts per workgroup (4 or 8)
    int q_blocks;     // shared kernel: blocks of shared_waves * shared_nq query tiles
    int ksplit_nq;    // 0, or 1 / 2: key-split kernel (wavefronts of a workgroup share the keys), query tiles per item
    int ksplit_waves; // key-split kernel: wavefronts per workgroup (4 or 8)
    int q_groups;     // key-split kernel: groups of ksplit_nq query tiles
};
AttnPlan dkv_attn_plan(int dtype, int batch, int n_q_heads, int n_kv_heads, int seq_len, int head_dim,
                       int max_rows_per_seq);
size_t dkv_attn_partial_bytes(const AttnPlan &p, int batch, int n_q_heads, int n_kv_heads, int head_dim);

// New K/V rows that the attention kernel itself writes into the cache before using them (all null: the cache
// is already up to date). Row r holds [n_kv_heads][head_dim] for position active_idx[r] of its sequence.
struct AttnFusedUpdate {
    const void *k_new, *v_new;
    const int *active_idx;
};
int dkv_attn_can_fuse_update(const AttnPlan &plan, int max_rows_per_seq);

// out[r, h, :] = attention of q[r, h] over all seq_len positions of sequence b(r).
int dkv_launch_attention(int dtype, const void *q, void *k_cache, void *v_cache, const int *row_off, void *out,
                         int batch, int n_q_heads, int n_kv_heads, int seq_len, int head_dim, int rows_upper,
                         AttnPlan plan, void *partial, AttnFusedUpdate fuse, hipStream_t stream);
