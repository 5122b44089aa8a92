// Translation unit of the guarded MFMA kernel (see kernels.hpp).
#include "kernels.hpp"
#include "gemm_edge.hpp"

namespace axonn {

void edge_kernel_raise_lds_limit() {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_edge_kernel<true, false>), hipFuncAttributeMaxDynamicSharedMemorySize, EdgeCfg::LDS_BYTES);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_edge_kernel<true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, EdgeCfg::LDS_BYTES);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_edge_kernel<false, false>), hipFuncAttributeMaxDynamicSharedMemorySize, EdgeCfg::LDS_BYTES);
}

void edge_kernel_launch(int layout, unsigned workgroups, hipStream_t s, const uint16_t* A, const uint16_t* B, uint16_t* C,
                        int64_t m, int64_t n, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int tiles_n) {
    const dim3 grid(workgroups), block(EdgeCfg::NT);
    switch (layout) {
        case 0:  hipLaunchKernelGGL((gemm_edge_kernel<true, false>), grid, block, EdgeCfg::LDS_BYTES, s, A, B, C, m, n, K, lda, ldb, ldc, tiles_n); break;
        case 1:  hipLaunchKernelGGL((gemm_edge_kernel<true, true>), grid, block, EdgeCfg::LDS_BYTES, s, A, B, C, m, n, K, lda, ldb, ldc, tiles_n); break;
        default: hipLaunchKernelGGL((gemm_edge_kernel<false, false>), grid, block, EdgeCfg::LDS_BYTES, s, A, B, C, m, n, K, lda, ldb, ldc, tiles_n); break;
    }
}

}  // namespace axonn
