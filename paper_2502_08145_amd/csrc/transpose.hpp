// Re-storing a bf16 operand for another GEMM mode (paper Sec. IV-C: NN, NT and TN differ only in how
// each operand lies in memory): dst[c * rows + r] = src[r * cols + c], 16-bit elements, bits moved.
//
// HBM-bound: 2 bytes read and 2 bytes written per element, nothing else.  The tile kernel moves a
// 64 x 64 tile per workgroup: 16-byte global loads of whole 128-byte row segments into LDS (row
// stride 144 bytes, which keeps the reads below conflict-free), then the transposing LDS read
// ds_read_b64_tr_b16 -- a 16-lane group turns a 4-row x 16-column block into, per lane, one column's
// four consecutive rows -- twice per lane for eight consecutive rows, i.e. 16 bytes of one output
// row, stored with one 16-byte global store.  A wave writes 16 output rows x 64 bytes per store and
// the two stores of a wave complete each 128-byte line.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace axonn {

typedef uint32_t tr_u32x4 __attribute__((ext_vector_type(4)));
typedef short tr_v4i16 __attribute__((ext_vector_type(4)));

constexpr int TR_TILE = 64;          // rows and columns per workgroup
constexpr int TR_LDS_STRIDE = 144;   // bytes per tile row in LDS (128 + 16)

// Requires rows % 64 == 0, cols % 64 == 0, both pointers 16-byte aligned.  grid = tiles, block = 256.
__global__ __launch_bounds__(256) void transpose_tile_kernel(const uint16_t* __restrict__ src,
                                                             uint16_t* __restrict__ dst, int64_t rows,
                                                             int64_t cols, int tiles_c) {
    __shared__ __attribute__((aligned(16))) uint8_t tile[TR_TILE * TR_LDS_STRIDE];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int64_t r0 = (int64_t)(blockIdx.x / tiles_c) * TR_TILE, c0 = (int64_t)(blockIdx.x % tiles_c) * TR_TILE;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int q = t + 256 * u, row = q >> 3, ch = q & 7;   // 16-byte chunk ch of tile row `row`
        const tr_u32x4 v = *reinterpret_cast<const tr_u32x4*>(src + (r0 + row) * cols + c0 + ch * 8);
        *reinterpret_cast<tr_u32x4*>(tile + row * TR_LDS_STRIDE + ch * 16) = v;
    }
    __syncthreads();
    // wave w owns tile columns 16w .. 16w+15 (16 output rows); lane = 16 g + s
    const int g = lane >> 4, s = lane & 15;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        // the group reads tile rows rb*32 + 8g + 0..3 (then + 4..7); lane s supplies row s>>2,
        // columns 16w + 4*(s&3) .. +3, and receives column 16w + s
        const uint8_t* p = tile + (rb * 32 + 8 * g + (s >> 2)) * TR_LDS_STRIDE + (16 * wave + 4 * (s & 3)) * 2;
        typedef __attribute__((address_space(3))) tr_v4i16 lds_v4i16;
        const tr_v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(p));
        const tr_v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(p + 4 * TR_LDS_STRIDE));
        tr_u32x4 out;
        out[0] = __builtin_bit_cast(uint32_t, __builtin_shufflevector(lo, lo, 0, 1));
        out[1] = __builtin_bit_cast(uint32_t, __builtin_shufflevector(lo, lo, 2, 3));
        out[2] = __builtin_bit_cast(uint32_t, __builtin_shufflevector(hi, hi, 0, 1));
        out[3] = __builtin_bit_cast(uint32_t, __builtin_shufflevector(hi, hi, 2, 3));
        *reinterpret_cast<tr_u32x4*>(dst + (c0 + 16 * wave + s) * rows + r0 + rb * 32 + 8 * g) = out;
    }
}

// Any rows, cols >= 1: one element per thread (stores coalesced along the output rows).
__global__ __launch_bounds__(256) void transpose_naive_kernel(const uint16_t* __restrict__ src,
                                                              uint16_t* __restrict__ dst, int64_t rows,
                                                              int64_t cols) {
    const int64_t r = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
    const int64_t c = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
    if (r < rows && c < cols) dst[c * rows + r] = src[r * cols + c];
}

}  // namespace axonn
