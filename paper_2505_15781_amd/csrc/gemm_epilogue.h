// Epilogues of the projection kernel: what a row kernel would do after re-reading the product happens on the
// accumulators instead (included by gemm_kernel.h inside its namespace). Only epilogues without loads are here (see
// the note at GemmEpilogue).
//
// Accumulator layout (MFMA 32x32x16, wave (wm, wn) of the workgroup tile at (m0, n0)): acc[i][j][v] is the
// element at column n0 + (wn NT + j) 32 + (lane & 31), row m0 + (wm MT + i) 32 + 8 (v >> 2) + 4 (lane >> 5) + (v & 3).
// So the 32 lanes of a half-wave hold 32 consecutive columns of one row, neighbouring lanes neighbouring columns.
#pragma once

// value of the neighbouring lane (lane ^ 1)
__device__ __forceinline__ float lane_swap1(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
}
// reductions over the 32 lanes that hold one row
__device__ __forceinline__ float half_sum(float v) {
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float half_max(float v) {
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ int half_min(int v) {
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) v = min(v, __shfl_xor(v, o, 64));
    return v;
}

// LDS scratch of the epilogues, carved out of the (now idle) tile stages.
template <int BM, int WN> struct EpiSmem {
    float red[BM][WN];       // EPI_HEAD: maxima of a row over each wavefront's columns
    float red2[BM][WN];      //           sums of exp(x - max)
    int redi[BM][WN];        //           arg maxima
};

template <int EPI, int MT, int NT, int WM, int WN>
__device__ __forceinline__ void run_epilogue(f32x16 (&acc)[MT][NT], const GemmEpilogue &ep, void *smem_raw,
                                             int m0, int n0, int M, int N, int tile_n, int tiles_n) {
    constexpr int BM = 32 * MT * WM, NW = WM * WN, NTHREADS = 64 * NW;
    EpiSmem<BM, WN> &sm = *reinterpret_cast<EpiSmem<BM, WN> *>(smem_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int col = lane & 31, rsub = 4 * (lane >> 5);

    if constexpr (EPI == EPI_SWIGLU) {
        // columns 2j (gate_j) and 2j+1 (up_j) sit in neighbouring lanes; even lanes finish accumulator elements
        // 0..7 and odd lanes 8..15, so every lane runs half of the activations
        bf16_t *f = static_cast<bf16_t *>(ep.out);
        const int F = N >> 1;
        const bool odd = lane & 1;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = (wm * MT + i) * 32 + 8 * (v >> 2) + rsub + (v & 3), m = m0 + r;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int n = n0 + (wn * NT + j) * 32 + col;
                    const float own = acc[i][j][v];
                    const float other = lane_swap1(own);
                    if ((v < 8) != odd) {
                        const float g = odd ? other : own, u = odd ? own : other;
                        const float y = g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;
                        if (m < M && n < N) f[(size_t)m * F + (n >> 1)] = f2bf(y);
                    }
                }
            }
    } else {   // EPI_HEAD
        float *logits = static_cast<float *>(ep.out);
        bool nan = false;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = (wm * MT + i) * 32 + 8 * (v >> 2) + rsub + (v & 3), m = m0 + r;
                float x[NT];
                float mx = -INFINITY;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int n = n0 + (wn * NT + j) * 32 + col;
                    x[j] = acc[i][j][v];
                    if (logits && m < M && n < N) logits[(size_t)m * N + n] = x[j];
                    if (n >= N || n == ep.mask_id) x[j] = -INFINITY;      // MASK can never be predicted
                    nan |= (x[j] != x[j]) && m < M;
                    mx = fmaxf(mx, x[j]);
                }
                mx = half_max(mx);
                float sum = 0.f;
                int best = 0x7fffffff;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int n = n0 + (wn * NT + j) * 32 + col;
                    if (x[j] > -INFINITY) sum += __expf(x[j] - mx);
                    if (x[j] == mx && mx > -INFINITY) best = min(best, n);      // lowest id on ties
                }
                sum = half_sum(sum);
                best = half_min(best);
                if (col == 0) {
                    sm.red[r][wn] = mx;
                    sm.red2[r][wn] = sum;
                    sm.redi[r][wn] = best;
                }
            }
        if (__any(nan) && lane == 0) atomicOr(ep.status, 1 /* STATUS_NAN */);
        __syncthreads();
        for (int r = tid; r < BM; r += NTHREADS) {
            const int m = m0 + r;
            if (m < M) {
                float mx = sm.red[r][0], sum = sm.red2[r][0];
                int best = sm.redi[r][0];
#pragma unroll
                for (int w = 1; w < WN; ++w) {      // ascending columns: ties keep the lower id
                    const float om = sm.red[r][w], os = sm.red2[r][w];
                    if (om > mx) {
                        sum = sum * __expf(mx - om) + os;      // mx == -inf only with sum == 0
                        mx = om;
                        best = sm.redi[r][w];
                    } else if (om > -INFINITY) {
                        sum += os * __expf(om - mx);
                    }
                }
                ep.head_part[(size_t)m * ep.head_tiles + tile_n] = HeadPartial{mx, sum, best, 0};
            }
        }
    }
}
