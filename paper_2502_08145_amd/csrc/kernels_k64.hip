// Translation unit of the 256 x 256 tile kernels with 64-k LDS stages (see kernels.hpp).
#include "kernels.hpp"
#include "gemm_mfma16_k64.hpp"
#include "gemm_mfma16_k64p.hpp"

namespace axonn {

tile_kernel_t k64_kernel(bool split, int layout) {
    static const tile_kernel_t fn[2][3] = {
        {gemm_tile_kernel_k64<4, true, false, false>, gemm_tile_kernel_k64<4, true, true, false>,
         gemm_tile_kernel_k64<4, false, false, false>},
        {gemm_tile_kernel_k64<4, true, false, true>, gemm_tile_kernel_k64<4, true, true, true>,
         gemm_tile_kernel_k64<4, false, false, true>},
    };
    return (layout >= 0 && layout < 3) ? fn[split ? 1 : 0][layout] : nullptr;
}

tile_kernel_t k64p_kernel(int layout) {
    static const tile_kernel_t fn[3] = {gemm_tile_kernel_k64p<true, false>, gemm_tile_kernel_k64p<true, true>,
                                        gemm_tile_kernel_k64p<false, false>};
    return (layout >= 0 && layout < 3) ? fn[layout] : nullptr;
}

}  // namespace axonn
