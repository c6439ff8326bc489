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
typedef __attribute__((address_space(3))) void *lds_ptr_t;

// 16 bytes per lane from global memory into LDS at lds_addr + 16 * lane (lds_addr wave-uniform).
// Issued through inline assembly so that the compiler does not serialise the ring on its own
// conservative wait; completion is awaited explicitly with vmcnt below.
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory", "m0");
}
// The same with the non-temporal hint: for weights that no other workgroup will read again (one row of tiles),
// so that they do not push the activations out of L2. Measured on cold weights: 5-11 % less time for the QKV
// and gate/up shapes at 16-128 rows; with several rows of tiles the hint costs up to 2x, hence the flag.
__device__ __forceinline__ void dma16_nt(const void *g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(g), "s"(lds_addr) : "memory", "m0");
}
// s_waitcnt immediate: vmcnt(n) [bits 3:0 and 15:14], lgkmcnt(0) when `lgkm0`, expcnt untouched
__device__ __forceinline__ constexpr int waitcnt_imm(int n, bool lgkm0) {
    return (n & 15) | ((n >> 4) << 14) | 0x0070 | (lgkm0 ? 0 : 0x0F00);
}

template <int MT, int NT, int WM, int WN, int STAGES>
__global__ __launch_bounds__(64 * WM * WN) void gemm_dma(const bf16_t *__restrict__ A,
                                                         const bf16_t *__restrict__ W, float *__restrict__ P,
                                                         int m_upper, int m_cap,
                                                         const int *__restrict__ m_dev, int N, int K,
                                                         int kt_per_split, int frac_units, int flags) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN, NW = WM * WN;
    constexpr int CA = BM / (8 * NW), CW = BN / (8 * NW);     // load instructions per thread per tile
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "whole load instructions per thread");
    constexpr int STAGE_CHUNKS = (BM + BN) * 8;
    static_assert((STAGES - 2) * (CA + CW) < 64, "vmcnt is a 6-bit counter");
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];

    const int M = m_dev ? min(*m_dev, m_upper) : m_upper;
    const int kt_total = K / BK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds_base = (uint32_t)(size_t)(lds_ptr_t)lds;

    // Work of this workgroup: one (tile, K slice) given by the 3-D grid, or, in fractional mode, the K-tile
    // units [w u, (w+1) u) of the sequence "tile 0's K tiles, tile 1's K tiles, ..." (tiles column-fastest),
    // which may end one output tile and begin the next. The part of tile t done by workgroup w goes to
    // partial slot w - floor(t * kt_total / u); the host only uses shares for which every tile gets the same
    // number of parts.
    const int tiles_n = (N + BN - 1) / BN;
    int unit = frac_units ? blockIdx.x * frac_units : 0;
    const int unit_end = frac_units ? min(unit + frac_units, tiles_n * ((m_upper + BM - 1) / BM) * kt_total) : 0;
  for (;;) {
    int m0, n0, kt0, nk, slot;
    if (frac_units) {
        const int tile = unit / kt_total;
        kt0 = unit - tile * kt_total;
        nk = min(kt_total - kt0, unit_end - unit);
        m0 = (tile / tiles_n) * BM;
        n0 = (tile % tiles_n) * BN;
        slot = blockIdx.x - (tile * kt_total) / frac_units;
        unit += nk;
    } else {
        int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
        if (flags & GEMM_FLAG_XCD_GROUP) {
            // position of this workgroup in the order "XCD 0's share, XCD 1's share, ..." of the sequence
            // (K slice, group of 4 tile rows, tile column, tile row within the group)
            const int gx = gridDim.x, gy = gridDim.y, total = gx * gy * gridDim.z;
            const int id = bx + gx * (by + gy * bz);
            // XCD x runs the ids x, x + 8, ...: total / 8 of them, one more for x < total % 8
            const int pos = (id & 7) * (total >> 3) + min(id & 7, total & 7) + (id >> 3);
            bz = pos / (gx * gy);
            const int p2 = pos - bz * gx * gy;
            const int grp = p2 / (4 * gx), within = p2 - grp * 4 * gx;
            const int rows_in_grp = min(4, gy - grp * 4);
            by = grp * 4 + within % rows_in_grp;
            bx = within / rows_in_grp;
        }
        m0 = by * BM;
        n0 = bx * BN;
        kt0 = bz * kt_per_split;
        nk = min(kt_total, kt0 + kt_per_split) - kt0;
        slot = bz;
    }
    if (m0 < M) {
    // first K tile of this workgroup's loop (the loop wraps around the slice)
    const int kt_rot = (flags & GEMM_FLAG_STAGGER) ? (int)((unsigned)(n0 / BN * 5 + m0 / BM * 3) % (unsigned)nk) : 0;

    // Source pointer of each load instruction for K tile kt0. Slot s of a stage holds row s/8, and in
    // position s%8 the chunk (s%8) ^ ((row>>1)&7). Rows past the end are clamped: they only feed outputs
    // that are never stored.
    const bf16_t *pa[CA], *pw[CW];
#pragma unroll
    for (int i = 0; i < CA; ++i) {
        int s = (i * NW + wave) * 64 + lane, row = s >> 3, kc = (s & 7) ^ ((row >> 1) & 7);
        pa[i] = A + (size_t)min(m0 + row, M - 1) * K + (size_t)kt0 * BK + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < CW; ++i) {
        int s = (i * NW + wave) * 64 + lane, row = s >> 3, kc = (s & 7) ^ ((row >> 1) & 7);
        pw[i] = W + (size_t)min(n0 + row, N - 1) * K + (size_t)kt0 * BK + kc * 8;
    }
    // Tiles past the slice are clamped to its last tile: the load count per step stays constant (so one
    // vmcnt value fits every iteration) and the redundant data lands in a stage nobody reads.
    auto issue = [&](int t, int stage) {
        int tt = min(t, nk - 1) + kt_rot;
        if (tt >= nk) tt -= nk;
        const size_t koff = (size_t)tt * BK;
        const uint32_t base = lds_base + (uint32_t)(stage * STAGE_CHUNKS + wave_u * 64) * 16u;
#pragma unroll
        for (int i = 0; i < CA; ++i) dma16(pa[i] + koff, base + (uint32_t)(i * NW * 64) * 16u);
        if (flags & GEMM_FLAG_STREAM_W) {
#pragma unroll
            for (int i = 0; i < CW; ++i) dma16_nt(pw[i] + koff, base + (uint32_t)(BM * 8 + i * NW * 64) * 16u);
        } else {
#pragma unroll
            for (int i = 0; i < CW; ++i) dma16(pw[i] + koff, base + (uint32_t)(BM * 8 + i * NW * 64) * 16u);
        }
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    bf16x8 af[2][MT], wf[2][NT];
    auto ldfrag = [&](int stage, int ks, int fb) {
        const bf16x8 *tile = reinterpret_cast<const bf16x8 *>(lds + stage * STAGE_CHUNKS);
        const int chunk = 2 * ks + (lane >> 5);
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            int row = (wm * MT + i) * 32 + (lane & 31);
            af[fb][i] = tile[row * 8 + (chunk ^ ((row >> 1) & 7))];
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            int row = (wn * NT + j) * 32 + (lane & 31);
            wf[fb][j] = tile[(BM + row) * 8 + (chunk ^ ((row >> 1) & 7))];
        }
    };
    // Make tile `next` readable: this wave's part of it has landed (all but the newest STAGES-2 tiles'
    // loads are done) and its own LDS reads have returned; after the barrier that holds for every wave, so
    // the stage read until now can be refilled and the first fragments of `next` fetched.
    auto advance = [&](int next) {
        __builtin_amdgcn_s_waitcnt(waitcnt_imm((STAGES - 2) * (CA + CW), true));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue(next + STAGES - 1, (next + STAGES - 1) % STAGES);
        ldfrag(next % STAGES, 0, 0);
    };

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(s, s);
    advance(0);
    for (int t = 0; t < nk; ++t) {
        const int stage = t % STAGES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) ldfrag(stage, ks + 1, (ks + 1) & 1);
            else if (t + 1 < nk) advance(t + 1);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], wf[ks & 1][j], acc[i][j], 0, 0, 0);
        }
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, false));   // the clamped tail loads must land before LDS is reused

    if (flags & GEMM_FLAG_SWIGLU) {
        // Fused SwiGLU (single K slice only): output columns 2j (gate_j) and 2j+1 (up_j) sit in neighbouring
        // lanes; each lane fetches its neighbour's value with a DPP quad permute, even lanes finish
        // accumulator elements 0..7 and odd lanes 8..15, and f[m][j] = silu(gate) * up goes out as bf16.
        bf16_t *f = reinterpret_cast<bf16_t *>(P);
        const int F = N >> 1;
        const bool odd = lane & 1;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int n = n0 + (wn * NT + j) * 32 + (lane & 31);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float own = acc[i][j][v];
                    const float other = __builtin_bit_cast(
                        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, own), 0xB1, 0xF, 0xF, true));
                    if ((v < 8) != odd) {
                        const float g = odd ? other : own, u = odd ? own : other;
                        const float r = g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;
                        const int m = m0 + (wm * MT + i) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                        if (m < M && n < N) f[(size_t)m * F + (n >> 1)] = f2bf(r);
                    }
                }
            }
    } else {
    float *out = P + (size_t)slot * m_cap * N;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int n = n0 + (wn * NT + j) * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + (wm * MT + i) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (m < M && n < N) out[(size_t)m * N + n] = acc[i][j][v];
            }
        }
    }
    }   // m0 < M
    if (!frac_units || unit >= unit_end) break;
    __syncthreads();      // every wave is done with the LDS stages before the next part refills them
  }
}

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
};
static_assert(sizeof(kKinds) / sizeof(kKinds[0]) == GEMM_DMA_256x192 + 1, "one entry per gemm_dma kind");


template <int MT, int NT, int WM, int WN, int STAGES>
int launch_dma(const void *A, const void *W, float *P, int m_upper, int m_cap, const int *m_dev, int n, int k,
               int split, int frac_units, int flags, hipStream_t s) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    constexpr int smem = STAGES * (BM + BN) * 128;
    // set once per process; the call is idempotent, so threads that race here only repeat it
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_dma<MT, NT, WM, WN, STAGES>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        attr_set.store(true, std::memory_order_release);
    }
    const int kt_total = k / BK, kps = ceil_div(kt_total, split);
    dim3 grid(ceil_div(n, BN), ceil_div(m_upper, BM), ceil_div(kt_total, kps));
    if (frac_units) {
        grid = dim3(ceil_div(grid.x * grid.y * kt_total, frac_units), 1, 1);
        if (flags & GEMM_FLAG_SWIGLU) {
            dkv_set_error("the fused SwiGLU epilogue needs one K slice");
            return DKV_E_INVALID_ARG;
        }
        flags = 0;
    }
    if (grid.y < 4) flags &= ~GEMM_FLAG_XCD_GROUP;
    if (grid.y > 1) flags &= ~GEMM_FLAG_STREAM_W;          // every weight tile is read once per row of tiles
    if ((flags & GEMM_FLAG_SWIGLU) && (grid.z != 1 || (n & 1))) {
        dkv_set_error("the fused SwiGLU epilogue needs one K slice and an even number of columns");
        return DKV_E_INVALID_ARG;
    }
    hipLaunchKernelGGL((gemm_dma<MT, NT, WM, WN, STAGES>), grid, dim3(64 * WM * WN), smem, s, (const bf16_t *)A,
                       (const bf16_t *)W, P, m_upper, m_cap, m_dev, n, k, kps, frac_units, flags);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

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
    for (int kind = 0; kind <= GEMM_DMA_256x192; ++kind) {
        const KindInfo &ki = kKinds[kind];
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
            double t = rounds * (nk * t_tile + kPipeFill);
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
    if (((p.kind == GEMM_DMA_256x256 || p.kind == GEMM_DMA_256x192) && tiles_m >= 4) ||
        (p.kind == GEMM_DMA_128x256 && tiles_m >= 6))
        p.flags |= GEMM_FLAG_XCD_GROUP;
    // Giving 256 workgroups 3/4 of a tile's K range each (frac_units, kept for experiments through
    // dkv_gemm_with) was measured to take the same time as two full slices, so it is never planned.
    return p;
}

bool dkv_gemm_can_fuse_swiglu(int dtype, int n, int k, const GemmPlan &p) {
    return dtype == DKV_BF16 && p.kind <= GEMM_DMA_256x192 && p.split_k == 1 && p.frac_units == 0 && (k % BK) == 0 &&
           (n & 1) == 0;
}

int dkv_gemm_plan_valid(int dtype, int k, GemmPlan p) {
    if (p.split_k < 1 || p.kind < 0 || p.kind >= GEMM_KINDS || p.frac_units < 0) return 0;
    if (p.frac_units) {
        // a 3/4 share: every tile is covered by exactly two workgroups
        if (p.kind > GEMM_DMA_256x192 || dtype != DKV_BF16 || (k % BK) != 0) return 0;
        return p.split_k == 2 && (k / BK) % 4 == 0 && p.frac_units == (k / BK) * 3 / 4;
    }
    if (p.kind == GEMM_SIMT) return p.split_k == 1;
    if (dtype != DKV_BF16 || (k % 8) != 0) return 0;
    if (p.kind != GEMM_REG_64x128 && (k % BK) != 0) return 0;
    return effective_split(k, p.split_k) == p.split_k;
}

int dkv_launch_gemm(int dtype, const void *A, const void *W, float *partial, int m_upper, int m_cap,
                    const int *m_dev, int n, int k, GemmPlan p, hipStream_t stream) {
    if (m_upper <= 0) return DKV_OK;
    if (!dkv_gemm_plan_valid(dtype, k, p)) {
        dkv_set_error("projection plan (kind %d, split %d) does not fit dtype %d, K %d", p.kind, p.split_k, dtype, k);
        return DKV_E_UNSUPPORTED;
    }
    switch (p.kind) {
        case GEMM_DMA_32x128:
            return launch_dma<1, 1, 1, 4, 4>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, stream);
        case GEMM_DMA_64x128:
            return launch_dma<2, 1, 1, 4, 4>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, stream);
        case GEMM_DMA_128x128:
            return launch_dma<2, 2, 2, 2, 3>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, stream);
        case GEMM_DMA_128x256:
            return launch_dma<2, 4, 2, 2, 3>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, stream);
        case GEMM_DMA_256x256:
            return launch_dma<4, 4, 2, 2, 2>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, stream);
        case GEMM_DMA_128x96:
            return launch_dma<1, 3, 4, 1, 4>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, stream);
        case GEMM_DMA_128x192:
            return launch_dma<2, 3, 2, 2, 3>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, stream);
        case GEMM_DMA_256x192:
            return launch_dma<4, 3, 2, 2, 2>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, stream);
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
