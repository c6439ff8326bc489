// The tile kernel of the projections (bf16, K a multiple of 64) and its launcher, as templates: one translation
// unit per epilogue instantiates them (gemm_epi_*.hip), so that the epilogues neither share registers nor
// compile in sequence. See gemm.hip for the design of the main loop.
#pragma once
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

#include "gemm_epilogue.h"

template <int EPI, int MT, int NT, int WM, int WN, int STAGES>
__global__ __launch_bounds__(64 * WM * WN) void gemm_dma(const bf16_t *__restrict__ A,
                                                         const bf16_t *__restrict__ W, float *__restrict__ P,
                                                         int m_upper, int m_cap,
                                                         const int *__restrict__ m_dev, int N, int K,
                                                         int kt_per_split, int frac_units, int flags,
                                                         const GemmEpilogue ep) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN, NW = WM * WN;
    constexpr int CA = BM / (8 * NW), CW = BN / (8 * NW);     // load instructions per thread per tile
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "whole load instructions per thread");
    constexpr int STAGE_CHUNKS = (BM + BN) * 8;
    static_assert((STAGES - 2) * (CA + CW) < 64, "vmcnt is a 6-bit counter");
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    static_assert(sizeof(EpiSmem<BM, WN>) <= STAGES * STAGE_CHUNKS * 16, "epilogue scratch fits the tile stages");

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

    if constexpr (EPI == EPI_STORE) {
        // every K slice leaves its sums in its own slot for the row kernel that consumes the product to add up
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
    } else {
        __syncthreads();                 // every wave is done with the tile stages: they become epilogue scratch
        run_epilogue<EPI, MT, NT, WM, WN>(acc, ep, lds, m0, n0, M, N, n0 / BN, tiles_n);
    }
    }   // m0 < M
    if (!frac_units || unit >= unit_end) break;
    __syncthreads();      // every wave is done with the LDS stages before the next part refills them
  }
}

template <int EPI, int MT, int NT, int WM, int WN, int STAGES>
int launch_dma(const void *A, const void *W, float *P, int m_upper, int m_cap, const int *m_dev, int n, int k,
               int split, int frac_units, int flags, const GemmEpilogue &ep, hipStream_t s) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    constexpr int smem = STAGES * (BM + BN) * 128;
    // set once per process; the call is idempotent, so threads that race here only repeat it
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        DKV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_dma<EPI, MT, NT, WM, WN, STAGES>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        attr_set.store(true, std::memory_order_release);
    }
    const int kt_total = k / BK, kps = ceil_div(kt_total, split);
    dim3 grid(ceil_div(n, BN), ceil_div(m_upper, BM), ceil_div(kt_total, kps));
    if (frac_units) {
        grid = dim3(ceil_div(grid.x * grid.y * kt_total, frac_units), 1, 1);
        flags = 0;
    }
    if (EPI != EPI_STORE && (frac_units || grid.z != 1)) {
        dkv_set_error("a fused epilogue needs one K slice");
        return DKV_E_INVALID_ARG;
    }
    if (grid.y < 4) flags &= ~GEMM_FLAG_XCD_GROUP;
    if (grid.y > 1) flags &= ~GEMM_FLAG_STREAM_W;          // every weight tile is read once per row of tiles
    if (EPI == EPI_SWIGLU && (n & 1)) {
        dkv_set_error("the fused SwiGLU epilogue pairs neighbouring columns: their number must be even");
        return DKV_E_INVALID_ARG;
    }
    hipLaunchKernelGGL((gemm_dma<EPI, MT, NT, WM, WN, STAGES>), grid, dim3(64 * WM * WN), smem, s, (const bf16_t *)A,
                       (const bf16_t *)W, P, m_upper, m_cap, m_dev, n, k, kps, frac_units, flags, ep);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}


template <int EPI>
int dispatch_dma(const void *A, const void *W, float *partial, int m_upper, int m_cap, const int *m_dev, int n, int k,
                 const GemmPlan &p, const GemmEpilogue &ep, hipStream_t stream) {
    switch (p.kind) {
        case GEMM_DMA_32x128:
            return launch_dma<EPI, 1, 1, 1, 4, 4>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
        case GEMM_DMA_64x128:
            return launch_dma<EPI, 2, 1, 1, 4, 4>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
        case GEMM_DMA_128x128:
            return launch_dma<EPI, 2, 2, 2, 2, 3>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
        case GEMM_DMA_128x256:
            return launch_dma<EPI, 2, 4, 2, 2, 3>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
        case GEMM_DMA_256x256:
            return launch_dma<EPI, 4, 4, 2, 2, 2>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
        case GEMM_DMA_128x96:
            return launch_dma<EPI, 1, 3, 4, 1, 4>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
        case GEMM_DMA_128x192:
            return launch_dma<EPI, 2, 3, 2, 2, 3>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
        case GEMM_DMA_256x192:
            return launch_dma<EPI, 4, 3, 2, 2, 2>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
        case GEMM_DMA_192x256:
            return launch_dma<EPI, 3, 4, 2, 2, 2>(A, W, partial, m_upper, m_cap, m_dev, n, k, p.split_k, p.frac_units, p.flags, ep, stream);
    }
    dkv_set_error("kernel %d is not a tile kernel", p.kind);
    return DKV_E_UNSUPPORTED;
}


}  // namespace
