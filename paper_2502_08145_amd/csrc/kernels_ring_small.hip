// Translation unit of the smaller tiles on the 32-k LDS ring (see kernels.hpp).
#include "kernels.hpp"
#include "gemm_mfma16.hpp"

namespace axonn {

#define AXONN_RING3(BM, BN, WN, SPLIT)                                                        \
    {gemm_tile_kernel16<BM, BN, 2, WN, true, false, SPLIT>, gemm_tile_kernel16<BM, BN, 2, WN, true, true, SPLIT>, \
     gemm_tile_kernel16<BM, BN, 2, WN, false, false, SPLIT>}

tile_kernel_t ring_kernel_small(int bm, int bn, int wn, bool split, int layout) {
    static const tile_kernel_t k256x128[3] = AXONN_RING3(256, 128, 2, false);
    static const tile_kernel_t k128x256[3] = AXONN_RING3(128, 256, 2, false);
    static const tile_kernel_t k128x256_w8[3] = AXONN_RING3(128, 256, 4, false);
    static const tile_kernel_t k256x128_sk[3] = AXONN_RING3(256, 128, 2, true);
    static const tile_kernel_t k128x256_sk[3] = AXONN_RING3(128, 256, 2, true);
    static const tile_kernel_t k128x128[3] = AXONN_RING3(128, 128, 2, false);
    static const tile_kernel_t k128x128_sk[3] = AXONN_RING3(128, 128, 2, true);
    if (layout < 0 || layout > 2) return nullptr;
    if (bm == 256 && bn == 128 && wn == 2) return (split ? k256x128_sk : k256x128)[layout];
    if (bm == 128 && bn == 256 && wn == 2) return (split ? k128x256_sk : k128x256)[layout];
    if (bm == 128 && bn == 256 && wn == 4 && !split) return k128x256_w8[layout];
    if (bm == 128 && bn == 128 && wn == 2) return (split ? k128x128_sk : k128x128)[layout];
    return nullptr;
}

}  // namespace axonn
