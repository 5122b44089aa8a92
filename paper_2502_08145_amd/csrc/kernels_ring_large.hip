// Translation unit of the 256 x 256 tile kernels on the 32-k LDS ring (see kernels.hpp).
#include "kernels.hpp"
#include "gemm_mfma16.hpp"

namespace axonn {

tile_kernel_t ring_kernel_large(bool split, int layout) {
    static const tile_kernel_t fn[2][3] = {
        {gemm_tile_kernel16<256, 256, 2, 4, true, false, false>, gemm_tile_kernel16<256, 256, 2, 4, true, true, false>,
         gemm_tile_kernel16<256, 256, 2, 4, false, false, false>},
        {gemm_tile_kernel16<256, 256, 2, 4, true, false, true>, gemm_tile_kernel16<256, 256, 2, 4, true, true, true>,
         gemm_tile_kernel16<256, 256, 2, 4, false, false, true>},
    };
    return (layout >= 0 && layout < 3) ? fn[split ? 1 : 0][layout] : nullptr;
}

}  // namespace axonn
