// The projection tile kernels with the EPI_STORE epilogue (see gemm_kernel.h, gemm_epilogue.h).
#include "gemm_kernel.h"

int dkv_dispatch_dma_store(const void *A, const void *W, float *partial, int m_upper, int m_cap, const int *m_dev, int n,
                         int k, const GemmPlan &plan, const GemmEpilogue &ep, hipStream_t stream) {
    return dispatch_dma<EPI_STORE>(A, W, partial, m_upper, m_cap, m_dev, n, k, plan, ep, stream);
}
