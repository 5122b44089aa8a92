// Translation unit of the 256 x 256 tile kernels with 64-k LDS stages (see kernels.hpp).
#include "kernels.hpp"
#include "gemm_mfma16_k64.hpp"
#include "gemm_mfma16_k64p.hpp"

namespace axonn {

// Load schedule per mode (see gemm_tile_kernel_k64): with two K-contiguous operands (NT) the A panel is
// triple-buffered and fetched in sub-step 0, measured 3-5 % faster at K of 4096 and more (2048 x 16384 x 4096:
// 1320 -> 1390 TFLOP/s, 8192^3: 1465 -> 1512) and no slower elsewhere; with an MN-contiguous operand it
// makes no difference (NN) or costs 2-5 % (TN, either operand triple-buffered), so those keep two buffers each.
constexpr int kSchedNN = 0, kSchedNT = 1, kSchedTN = 0;

tile_kernel_t k64_kernel(bool split, int layout) {
    static const tile_kernel_t fn[2][3] = {
        {gemm_tile_kernel_k64<256, 256, 4, true, false, false, kSchedNN>, gemm_tile_kernel_k64<256, 256, 4, true, true, false, kSchedNT>,
         gemm_tile_kernel_k64<256, 256, 4, false, false, false, kSchedTN>},
        {gemm_tile_kernel_k64<256, 256, 4, true, false, true, kSchedNN>, gemm_tile_kernel_k64<256, 256, 4, true, true, true, kSchedNT>,
         gemm_tile_kernel_k64<256, 256, 4, false, false, true, kSchedTN>},
    };
    return (layout >= 0 && layout < 3) ? fn[split ? 1 : 0][layout] : nullptr;
}

// The 64-k kernel on the half tiles: four waves (2 x 2), three buffers per operand (144 KB), half of an
// iteration's loads in either sub-step.  NT only: there it measures 28 % over the 32-k ring on the same
// tiles (2048 x 4096 x 4096: 1018 against 794 TFLOP/s; 4096^3: 1141 against 949); with an MN-contiguous
// operand it is 15-30 % BEHIND the ring (NN 743 against 990, TN 704 against 904), like every schedule
// tried that issues such an operand's loads anywhere but straight after the barrier.
tile_kernel_t k64_kernel_half(int bm, int bn, bool split, int layout) {
    if (layout != 1) return nullptr;
    if (bm == 256 && bn == 128)
        return split ? gemm_tile_kernel_k64<256, 128, 2, true, true, true, 3> : gemm_tile_kernel_k64<256, 128, 2, true, true, false, 3>;
    if (bm == 128 && bn == 256)
        return split ? gemm_tile_kernel_k64<128, 256, 2, true, true, true, 3> : gemm_tile_kernel_k64<128, 256, 2, true, true, false, 3>;
    return nullptr;
}

tile_kernel_t k64p_kernel(int layout) {
    static const tile_kernel_t fn[3] = {gemm_tile_kernel_k64p<true, false>, gemm_tile_kernel_k64p<true, true>,
                                        gemm_tile_kernel_k64p<false, false>};
    return (layout >= 0 && layout < 3) ? fn[layout] : nullptr;
}

}  // namespace axonn
