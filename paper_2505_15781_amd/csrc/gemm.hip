// Projection kernels: partial[s][m][n] = A[m, k-slice s] * W[n, k-slice s]^T, fp32 accumulation.
//
// The active rows of a denoising step (Algorithm 1 line 3: the transformer runs on x[M_{t-1}] only)
// are the M dimension; their count lives on the device, so kernels bound M by *m_dev.
//
// bf16, K a multiple of 64 (every model shape): `gemm_dma`. MFMA 32x32x16 tiles; the A and W tiles of
// a K step travel from global memory straight into LDS (global_load_lds_dwordx4: 16 bytes per lane, lane i
// lands at base + 16 i) through a ring of STAGES buffers, so up to STAGES-1 tiles are in flight without
// holding registers. The LDS layout XOR-swizzles the 16-byte chunks of a 128-byte row with (row >> 1)
// so a fragment read of 16 consecutive rows touches every bank once; the swizzle is applied by choosing
// which global chunk each lane fetches. Fragment reads run one K sub-step ahead of the MFMAs, across tile
// boundaries. Measured on MI355X a compute unit sustains about 60 GB/s of such fills whatever the depth,
// so the tile shapes below are chosen to keep the bytes each workgroup pulls (W tile + A tile) small
// relative to its MFMA work, and K is split across workgroups only as far as needed to fill 256 CUs.
// Two launch options, both measured: `stagger` starts each workgroup's K loop at a different tile (unsplit
// launches otherwise sweep the same columns of A and W in step and crowd a few memory channels: up to 25 %
// on the widest projection at <= 128 rows); `xcd_group` renumbers workgroups so that the 32 that run
// together on one XCD (hardware sends workgroup i to XCD i mod 8) cover a compact 4 x 8 block of tiles and
// share their A and W tiles through that XCD's L2 (hit rate 54 % -> 78 % and 5 % less time at 6144 rows).
// bf16, other K (multiple of 8): `gemm_reg`, register-staged tiles. fp32 mode / anything else: `gemm_simt`.
#include <atomic>

#include "common.h"

namespace {

constexpr int BK = 64;   // K elements per LDS tile (8 chunks of 8 bf16)

// Register-staged variant for K that is a multiple of 8 but not of 64 (zero-fills the K tail).
__global__ __launch_bounds__(256) void gemm_reg(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                                                float *__restrict__ P, int m_upper, int m_cap,
                                                const int *__restrict__ m_dev, int N, int K, int kt_per_split) {
    constexpr int MT = 2, BM = 64, BN = 128, CA = 2, CW = 4;
    __shared__ uint4 lds[2][(BM + BN) * 8];
    const int M = m_dev ? min(*m_dev, m_upper) : m_upper;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (m0 >= M) return;
    const int kt_total = (K + BK - 1) / BK;
    const int kt0 = blockIdx.z * kt_per_split, kt1 = min(kt_total, kt0 + kt_per_split);
    const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
    uint4 ra[CA], rw[CW];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            int c = tid + 256 * i, row = c >> 3, kc = c & 7, gm = m0 + row, gk = kt * BK + kc * 8;
            ra[i] = (gm < M && gk < K) ? *reinterpret_cast<const uint4 *>(A + (size_t)gm * K + gk) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            int c = tid + 256 * i, row = c >> 3, kc = c & 7, gn = n0 + row, gk = kt * BK + kc * 8;
            rw[i] = (gn < N && gk < K) ? *reinterpret_cast<const uint4 *>(W + (size_t)gn * K + gk) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            lds[buf][row * 8 + (kc ^ ((row >> 1) & 7))] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            lds[buf][(BM + row) * 8 + (kc ^ ((row >> 1) & 7))] = rw[i];
        }
    };
    f32x16 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    if (kt0 < kt1) {
        load_global(kt0);
        store_lds(0);
    }
    __syncthreads();
    for (int kt = kt0; kt < kt1; ++kt) {
        const int buf = (kt - kt0) & 1;
        if (kt + 1 < kt1) load_global(kt + 1);
        const bf16x8 *tile = reinterpret_cast<const bf16x8 *>(lds[buf]);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int chunk = 2 * ks + (lane >> 5);
            const int wrow = wn * 32 + (lane & 31);
            const bf16x8 wfr = tile[(BM + wrow) * 8 + (chunk ^ ((wrow >> 1) & 7))];
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const int row = i * 32 + (lane & 31);
                const bf16x8 afr = tile[row * 8 + (chunk ^ ((row >> 1) & 7))];
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afr, wfr, acc[i], 0, 0, 0);
            }
        }
        if (kt + 1 < kt1) store_lds(buf ^ 1);
        __syncthreads();
    }
    float *out = P + (size_t)blockIdx.z * m_cap * N;
    const int n = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (m < M && n < N) out[(size_t)m * N + n] = acc[i][v];
        }
}

// Plain FMA tile kernel: 64x64 outputs per workgroup, 4x4 per thread.
template <typename T>
__global__ __launch_bounds__(256) void gemm_simt(const T *__restrict__ A, const T *__restrict__ W,
                                                 float *__restrict__ P, int m_upper,
                                                 const int *__restrict__ m_dev, int N, int K) {
    constexpr int TM = 64, TN = 64, TK = 16;
    __shared__ float As[TK][TM + 4], Ws[TK][TN + 4];
    const int M = m_dev ? min(*m_dev, m_upper) : m_upper;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    if (m0 >= M) return;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    for (int kb = 0; kb < K; kb += TK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int e = tid + 256 * i, row = e >> 4, kk = e & 15;
            int gk = kb + kk;
            As[kk][row] = (m0 + row < M && gk < K) ? El<T>::ld(A + (size_t)(m0 + row) * K + gk) : 0.f;
            Ws[kk][row] = (n0 + row < N && gk < K) ? El<T>::ld(W + (size_t)(n0 + row) * K + gk) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) P[(size_t)m * N + n] = acc[i][j];
        }
}

struct KindInfo {
    int bm, bn;
};
constexpr KindInfo kKinds[] = {
    {32, 128},    // GEMM_DMA_32x128   <1,1,1,4> 4 stages
    {64, 128},    // GEMM_DMA_64x128   <2,1,1,4> 4 stages
    {128, 128},   // GEMM_DMA_128x128  <2,2,2,2> 3 stages
    {128, 256},   // GEMM_DMA_128x256  <2,4,2,2> 3 stages
    {256, 256},   // GEMM_DMA_256x256  <4,4,2,2> 2 stages
    {128, 96},    // GEMM_DMA_128x96   <1,3,4,1> 4 stages
    {128, 192},   // GEMM_DMA_128x192  <2,3,2,2> 3 stages
    {256, 192},   // GEMM_DMA_256x192  <4,3,2,2> 2 stages
    {192, 256},   // GEMM_DMA_192x256  <3,4,2,2> 2 stages
};
static_assert(sizeof(kKinds) / sizeof(kKinds[0]) == GEMM_DMA_LAST + 1, "one entry per gemm_dma kind");
static_assert(GEMM_DMA_192x256 == DKV_GEMM_DMA_192x256 && GEMM_REG_64x128 == DKV_GEMM_REG_64x128 &&
                  GEMM_SIMT == DKV_GEMM_SIMT && GEMM_KINDS == DKV_PROF_ATTN,
              "the kinds of the public header are these");

// Number of K slices that is really launched for a requested split (no empty slice).
int effective_split(int k, int split) {
    const int kt_total = ceil_div(k, BK), kps = ceil_div(kt_total, split < 1 ? 1 : split);
    return ceil_div(kt_total, kps);
}

}  // namespace

GemmPlan dkv_gemm_plan(int dtype, int m_upper, int n, int k) {
    GemmPlan p;
    p.split_k = 1;
    p.frac_units = 0;
    p.flags = 0;
    if (dtype != DKV_BF16 || (k % 8) != 0) {
        p.kind = GEMM_SIMT;
        return p;
    }
    if (k % BK != 0) {
        p.kind = GEMM_REG_64x128;
        return p;
    }
    // Tile shape and K split: the candidate with the smallest predicted launch time. The prediction is a
    // small model of this kernel on MI355X, its constants fitted to a sweep of every (tile shape, split)
    // over the layer shapes of the 8B and 7B models at 16..12288 rows (mean loss against the best measured
    // candidate 2 %, worst 24 %):
    //   a workgroup needs, per K tile, the longer of filling its LDS stage (~49 GB/s per compute unit, and
    //   ~14 TB/s over all workgroups in flight) and its MFMAs (~5.3 TFLOP/s per compute unit);
    //   workgroups run in rounds of 256 (one per compute unit), a partly filled round costs a full one;
    //   no launch beats streaming its operands and results once;
    //   K slices add the write and re-read of their partial sums by the consumer.
    // Tiles of 96 and 192 columns exist because 12288 / 96 = 128 and 24576 / 192 = 128 column tiles make
    // exactly one or two full rounds where 128- and 256-column tiles leave a quarter of the chip idle
    // (256x192 does the same for 257..512 rows of the widest projection).
    constexpr double kFillPerCu = 48785.0, kFlopsPerCu = 5332277.0, kFillAll = 14076233.0;   // bytes, flops per us
    constexpr double kStream = 7841520.0, kReduce = 1819886.0;                                  // bytes per us
    constexpr double kLaunch = 3.5, kPipeFill = 0.7, kReduceFixed = 1.7;                        // us
    static const int kSplits[] = {1, 2, 3, 4, 6, 8};
    const int kt_total = k / BK;
    double best = 0.0;
    p.kind = -1;
    for (int kind = 0; kind <= GEMM_DMA_LAST; ++kind) {
        const KindInfo &ki = kKinds[kind];
        // 192-row tiles are for thousands of rows, where 6144 = 32 x 192 rows against 4096 columns make two full
        // rounds of workgroups (128x256 tiles: three rounds of smaller tiles; 256x256: one and a half)
        if (kind == GEMM_DMA_192x256 && m_upper < 4 * ki.bm) continue;
        if (ki.bm > 32 && ki.bm >= 4 * m_upper) continue;       // mostly padding
        if (ki.bm < 128 && m_upper > 4 * ki.bm) continue;       // W re-read too often
        const int tiles = ceil_div(m_upper, ki.bm) * ceil_div(n, ki.bn);
        const double fill = (ki.bm + ki.bn) * 128.0, flops = 2.0 * ki.bm * ki.bn * BK;
        for (int s : kSplits) {
            const int nk = ceil_div(kt_total, s);
            if (ceil_div(kt_total, nk) != s || (s > 1 && nk < 8)) continue;
            const long wgs = (long)tiles * s;
            const long rounds = (wgs + 255) / 256;
            double t_tile = fill / kFillPerCu;
            if (flops / kFlopsPerCu > t_tile) t_tile = flops / kFlopsPerCu;
            const double in_flight = (double)(wgs < 256 ? wgs : 256);
            if (in_flight * fill / kFillAll > t_tile) t_tile = in_flight * fill / kFillAll;
            // (the 192x256 tile's fill and MFMA times are equal, so neither hides behind the other: measured 5 % above
            // the model where the 256x256 tile meets it)
            double t = rounds * (nk * t_tile * (kind == GEMM_DMA_192x256 ? 1.05 : 1.0) + kPipeFill);
            const double stream = (2.0 * n * k + 2.0 * m_upper * (double)k + 4.0 * s * m_upper * (double)n) / kStream;
            if (stream > t) t = stream;
            t += kLaunch;
            if (s > 1) t += (s + 1) * 4.0 * m_upper * (double)n / kReduce + kReduceFixed;
            if (p.kind < 0 || t < best) {
                best = t;
                p.kind = kind;
                p.split_k = s;
            }
        }
    }
    // Launch options, from the same sweep: a staggered K start pays when there is one row of tiles
    // (all workgroups of a K slice would otherwise read the same A columns at once); weights that are read once
    // (one row of tiles) are streamed with the non-temporal hint; the XCD-grouped order
    // pays for the largest tiles once there are enough tile rows to form 4-row groups.
    const int tiles_m = ceil_div(m_upper, kKinds[p.kind].bm);
    if (tiles_m == 1) p.flags |= GEMM_FLAG_STAGGER;
    // (not for matrices small enough to stay in the 256 MB last-level cache from one step to the next)
    if (tiles_m == 1 && (size_t)n * k * 2 >= ((size_t)32 << 20)) p.flags |= GEMM_FLAG_STREAM_W;
    if (((p.kind == GEMM_DMA_256x256 || p.kind == GEMM_DMA_256x192 || p.kind == GEMM_DMA_192x256) && tiles_m >= 4) ||
        (p.kind == GEMM_DMA_128x256 && tiles_m >= 6))
        p.flags |= GEMM_FLAG_XCD_GROUP;
    // Giving 256 workgroups 3/4 of a tile's K range each (frac_units, kept for experiments through
    // dkv_gemm_with) was measured to take the same time as two full slices, so it is never planned.
    return p;
}

bool dkv_gemm_can_fuse_swiglu(int dtype, int n, int k, const GemmPlan &p) {
    return dtype == DKV_BF16 && p.kind <= GEMM_DMA_LAST && p.split_k == 1 && p.frac_units == 0 && (k % BK) == 0 &&
           (n & 1) == 0;
}

int dkv_gemm_plan_valid(int dtype, int k, GemmPlan p) {
    if (p.split_k < 1 || p.kind < 0 || p.kind >= GEMM_KINDS || p.frac_units < 0) return 0;
    if (p.frac_units) {
        // a 3/4 share: every tile is covered by exactly two workgroups
        if (p.kind > GEMM_DMA_LAST || dtype != DKV_BF16 || (k % BK) != 0) return 0;
        return p.split_k == 2 && (k / BK) % 4 == 0 && p.frac_units == (k / BK) * 3 / 4;
    }
    if (p.kind == GEMM_SIMT) return p.split_k == 1;
    if (dtype != DKV_BF16 || (k % 8) != 0) return 0;
    if (p.kind != GEMM_REG_64x128 && (k % BK) != 0) return 0;
    return effective_split(k, p.split_k) == p.split_k;
}

bool dkv_gemm_can_fuse_head(int dtype, int k, const GemmPlan &p) {
    return dtype == DKV_BF16 && p.kind >= 0 && p.kind <= GEMM_DMA_LAST && p.split_k == 1 && p.frac_units == 0 &&
           (k % BK) == 0;
}

int dkv_gemm_tiles_n(const GemmPlan &p, int n) {
    return p.kind >= 0 && p.kind <= GEMM_DMA_LAST ? ceil_div(n, kKinds[p.kind].bn) : 0;
}

int dkv_launch_gemm_head(const void *A, const void *W, int m_upper, const int *m_dev, int n, int k, GemmPlan p,
                         const GemmEpilogue &ep, hipStream_t stream) {
    if (m_upper <= 0) return DKV_OK;
    if (ep.kind != EPI_HEAD || !dkv_gemm_can_fuse_head(DKV_BF16, k, p) || !dkv_gemm_plan_valid(DKV_BF16, k, p)) {
        dkv_set_error("projection plan (kind %d, split %d) cannot run the vocabulary epilogue at K %d", p.kind, p.split_k, k);
        return DKV_E_UNSUPPORTED;
    }
    p.flags &= ~GEMM_FLAG_SWIGLU;
    return dkv_dispatch_dma_head(A, W, nullptr, m_upper, m_upper, m_dev, n, k, p, ep, stream);
}

int dkv_launch_gemm(int dtype, const void *A, const void *W, float *partial, int m_upper, int m_cap,
                    const int *m_dev, int n, int k, GemmPlan p, hipStream_t stream) {
    if (m_upper <= 0) return DKV_OK;
    if (!dkv_gemm_plan_valid(dtype, k, p)) {
        dkv_set_error("projection plan (kind %d, split %d) does not fit dtype %d, K %d", p.kind, p.split_k, dtype, k);
        return DKV_E_UNSUPPORTED;
    }
    if (p.kind <= GEMM_DMA_LAST) {
        GemmEpilogue ep;
        if (p.flags & GEMM_FLAG_SWIGLU) {
            if (p.split_k != 1 || p.frac_units) {
                dkv_set_error("the fused SwiGLU epilogue of a plain launch needs one K slice");
                return DKV_E_INVALID_ARG;
            }
            ep.kind = EPI_SWIGLU;
            ep.out = partial;
            return dkv_dispatch_dma_swiglu(A, W, partial, m_upper, m_cap, m_dev, n, k, p, ep, stream);
        }
        return dkv_dispatch_dma_store(A, W, partial, m_upper, m_cap, m_dev, n, k, p, ep, stream);
    }
    switch (p.kind) {
        case GEMM_REG_64x128: {
            const int kt_total = ceil_div(k, BK), kps = ceil_div(kt_total, p.split_k);
            dim3 grid(ceil_div(n, 128), ceil_div(m_upper, 64), p.split_k);
            hipLaunchKernelGGL(gemm_reg, grid, dim3(256), 0, stream, (const bf16_t *)A, (const bf16_t *)W, partial,
                               m_upper, m_cap, m_dev, n, k, kps);
            break;
        }
        default: {
            dim3 grid(ceil_div(n, 64), ceil_div(m_upper, 64), 1);
            if (dtype == DKV_BF16)
                hipLaunchKernelGGL((gemm_simt<bf16_t>), grid, dim3(256), 0, stream, (const bf16_t *)A,
                                   (const bf16_t *)W, partial, m_upper, m_dev, n, k);
            else
                hipLaunchKernelGGL((gemm_simt<float>), grid, dim3(256), 0, stream, (const float *)A,
                                   (const float *)W, partial, m_upper, m_dev, n, k);
        }
    }
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}
