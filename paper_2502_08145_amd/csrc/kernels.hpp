// The GEMM kernels are compiled in several translation units (the compile time is theirs); this
// header is what the host side (axonn_linear.hip) sees of them: one look-up function per unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma.hpp"

namespace axonn {

// (A, B, C, K, lda, ldb, ldc, tiles_m, tiles_n, group_m, split-K state): leading dimensions in elements of
// the operands as stored, so that a launch can cover a block of rows or columns of a larger product
typedef void (*tile_kernel_t)(const uint16_t*, const uint16_t*, uint16_t*, int, int, int, int, int, int, int, SplitK);

// layout: 0 NN, 1 NT, 2 TN.  nullptr: no such kernel.
// 32-k LDS ring (gemm_tile_kernel16): tile bm x bn, 2 x wn waves, with or without split-K
tile_kernel_t ring_kernel_large(bool split, int layout);                          // 256 x 256, 2 x 4 waves
tile_kernel_t ring_kernel_small(int bm, int bn, int wn, bool split, int layout);  // 256x128, 128x256 (wn 2; wn 4 without split-K), 128x128
// 64-k stages (gemm_tile_kernel_k64): 256 x 256, 2 x 4 waves
tile_kernel_t k64_kernel(bool split, int layout);
// the same on 256 x 128 and 128 x 256 tiles, 2 x 2 waves, three LDS buffers per operand (NT only)
tile_kernel_t k64_kernel_half(int bm, int bn, bool split, int layout);
// the same with one resident workgroup per compute unit walking a list of tiles (gemm_tile_kernel_k64p)
tile_kernel_t k64p_kernel(int layout);

// guarded MFMA kernel (gemm_edge_kernel): any m, n, K >= 1 and any leading dimensions
void edge_kernel_raise_lds_limit();
void edge_kernel_launch(int layout, unsigned workgroups, hipStream_t s, const uint16_t* A, const uint16_t* B, uint16_t* C,
                        int64_t m, int64_t n, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int tiles_n);

}  // namespace axonn
