// Projection kernels: partial[s][m][n] = A[m, k-slice s] * W[n, k-slice s]^T, fp32 accumulation.
//
// bf16: MFMA 32x32x16 tiles, 256 threads (4 wavefronts) per workgroup, A and W tiles staged through
// LDS in 16-byte chunks (XOR-swizzled by row so fragment reads spread over the banks), global
// loads of the next K tile in flight while the current one is multiplied.
// fp32 (and any shape the MFMA kernel does not take): a plain FMA tile kernel.
//
// The active rows of a denoising step (Algorithm 1 line 3: the transformer runs on x[M_{t-1}] only)
// are the M dimension; their count lives on the device, so kernels bound M by *m_dev.
#include "common.h"

namespace {

constexpr int BK = 64;   // K elements per LDS tile (8 chunks of 8 bf16)

template <int MT, int NT, int WM, int WN>
__global__ __launch_bounds__(256) void gemm_bf16_mfma(const bf16_t *__restrict__ A,
                                                      const bf16_t *__restrict__ W,
                                                      float *__restrict__ P, int m_upper, int m_cap,
                                                      const int *__restrict__ m_dev, int N, int K,
                                                      int kt_per_split) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    constexpr int CA = BM / 32, CW = BN / 32;            // 16-byte chunks per thread per tile
    __shared__ uint4 lds[2][(BM + BN) * 8];

    const int M = m_dev ? min(*m_dev, m_upper) : m_upper;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (m0 >= M) return;
    const int kt_total = (K + BK - 1) / BK;
    const int kt0 = blockIdx.z * kt_per_split;
    const int kt1 = min(kt_total, kt0 + kt_per_split);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    uint4 ra[CA], rw[CW];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            int gm = m0 + row, gk = kt * BK + kc * 8;
            ra[i] = (gm < M && gk < K) ? *reinterpret_cast<const uint4 *>(A + (size_t)gm * K + gk)
                                       : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            int gn = n0 + row, gk = kt * BK + kc * 8;
            rw[i] = (gn < N && gk < K) ? *reinterpret_cast<const uint4 *>(W + (size_t)gn * K + gk)
                                       : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            lds[buf][row * 8 + (kc ^ (row & 7))] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            lds[buf][(BM + row) * 8 + (kc ^ (row & 7))] = rw[i];
        }
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

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
            bf16x8 af[MT], wf[NT];
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                int row = (wm * MT + i) * 32 + (lane & 31);
                af[i] = tile[row * 8 + (chunk ^ (row & 7))];
            }
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                int row = (wn * NT + j) * 32 + (lane & 31);
                wf[j] = tile[(BM + row) * 8 + (chunk ^ (row & 7))];
            }
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < kt1) store_lds(buf ^ 1);
        __syncthreads();
    }

    float *out = P + (size_t)blockIdx.z * m_cap * N;
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

// Plain FMA tile kernel: 64x64 outputs per workgroup, 4x4 per thread.
template <typename T>
__global__ __launch_bounds__(256) void gemm_simt(const T *__restrict__ A, const T *__restrict__ W,
                                                 float *__restrict__ P, int m_upper, int m_cap,
                                                 const int *__restrict__ m_dev, int N, int K,
                                                 int k_per_split) {
    constexpr int TM = 64, TN = 64, TK = 16;
    __shared__ float As[TK][TM + 4], Ws[TK][TN + 4];
    const int M = m_dev ? min(*m_dev, m_upper) : m_upper;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    if (m0 >= M) return;
    const int k0 = blockIdx.z * k_per_split, k1 = min(K, k0 + k_per_split);
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    for (int kb = k0; kb < k1; kb += TK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int e = tid + 256 * i, row = e >> 4, kk = e & 15;
            int gk = kb + kk;
            As[kk][row] = (m0 + row < M && gk < k1) ? El<T>::ld(A + (size_t)(m0 + row) * K + gk) : 0.f;
            Ws[kk][row] = (n0 + row < N && gk < k1) ? El<T>::ld(W + (size_t)(n0 + row) * K + gk) : 0.f;
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
    float *out = P + (size_t)blockIdx.z * m_cap * N;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) out[(size_t)m * N + n] = acc[i][j];
        }
}

template <int MT, int NT, int WM, int WN>
void launch_mfma(const void *A, const void *W, float *P, int m_upper, int m_cap, const int *m_dev, int n,
                 int k, int split, hipStream_t s) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    int kt_total = ceil_div(k, BK), kps = ceil_div(kt_total, split);
    dim3 grid(ceil_div(n, BN), ceil_div(m_upper, BM), ceil_div(kt_total, kps));
    hipLaunchKernelGGL((gemm_bf16_mfma<MT, NT, WM, WN>), grid, dim3(256), 0, s, (const bf16_t *)A,
                       (const bf16_t *)W, P, m_upper, m_cap, m_dev, n, k, kps);
}

}  // namespace

GemmPlan dkv_gemm_plan(int dtype, int m_upper, int n, int k) {
    GemmPlan p;
    if (dtype != DKV_BF16 || (k % 8) != 0) {
        p.bm = 64;
        p.split_k = 1;
        return p;
    }
    p.bm = m_upper <= 32 ? 32 : (m_upper <= 64 ? 64 : 128);
    int tiles = ceil_div(m_upper, p.bm) * ceil_div(n, 128);
    int kt_total = ceil_div(k, BK);
    int s = 1;
    if (tiles < 256) {
        s = ceil_div(512, tiles);
        int max_s = kt_total / 4 > 0 ? kt_total / 4 : 1;
        if (s > max_s) s = max_s;
        if (s > 16) s = 16;
    }
    int kps = ceil_div(kt_total, s);
    p.split_k = ceil_div(kt_total, kps);
    return p;
}

int dkv_launch_gemm(int dtype, const void *A, const void *W, float *partial, int m_upper, int m_cap,
                    const int *m_dev, int n, int k, GemmPlan plan, hipStream_t stream) {
    if (m_upper <= 0) return DKV_OK;
    if (dtype == DKV_BF16 && (k % 8) == 0) {
        if (plan.bm == 32)
            launch_mfma<1, 1, 1, 4>(A, W, partial, m_upper, m_cap, m_dev, n, k, plan.split_k, stream);
        else if (plan.bm == 64)
            launch_mfma<2, 1, 1, 4>(A, W, partial, m_upper, m_cap, m_dev, n, k, plan.split_k, stream);
        else
            launch_mfma<2, 2, 2, 2>(A, W, partial, m_upper, m_cap, m_dev, n, k, plan.split_k, stream);
    } else {
        dim3 grid(ceil_div(n, 64), ceil_div(m_upper, 64), 1);
        if (dtype == DKV_BF16)
            hipLaunchKernelGGL((gemm_simt<bf16_t>), grid, dim3(256), 0, stream, (const bf16_t *)A,
                               (const bf16_t *)W, partial, m_upper, m_cap, m_dev, n, k, k);
        else
            hipLaunchKernelGGL((gemm_simt<float>), grid, dim3(256), 0, stream, (const float *)A,
                               (const float *)W, partial, m_upper, m_cap, m_dev, n, k, k);
    }
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}
