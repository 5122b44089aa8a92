// Guarded MFMA kernel: the same product as the tile kernels,
//
//   C[M,N] = sum_k a(i,k) b(k,j)      (the local matrix multiply of Algorithm 1 lines 3, 11, 13)
//
// for ANY M, N, K >= 1 and any leading dimensions: ragged edges in all three directions, operand
// rows that are not 16-byte aligned.  It serves the shapes the tile kernels do not take (they want
// whole tiles and K in whole K-steps) and the edge strips that a plan cuts off a ragged output.
//
// Built for being right at every shape rather than for the last per cent:
//  * 128 x 128 output tile per workgroup of 4 waves (2 x 2, 64 x 64 per wave), K 128 at a time,
//    v_mfma_f32_16x16x32_bf16 with fp32 accumulators over all of K, one RNE rounding at the store.
//  * Operands go global -> registers -> LDS in 16-byte pieces of 8 elements along the operand's
//    contiguous dimension.  A piece that lies wholly inside the matrix at a 16-byte aligned address
//    is one vector load; any other piece is fetched element by element, and whatever lies outside
//    (rows or columns beyond the block, k beyond K) is zero, in BOTH operands, so that nothing
//    outside the product can reach an accumulator.  The loads of K-step t+1 are in flight while
//    step t is multiplied (one LDS buffer, two barriers per step).  The step is long because an
//    edge strip is often a single workgroup per compute unit, with nobody to hide the latency of
//    its loads behind: 32 k a step measured 1 us per step, whatever the step held.
//  * LDS holds a K-contiguous operand as rows of 128 k (256 bytes, padded to 272: conflict-free
//    ds_read_b128 fragments) and an MN-contiguous operand as it is in memory, one row per k (256
//    bytes, padded to 288), read with the transposing ds_read_b64_tr_b16.  No inline asm: the
//    compiler places the waits.
//  * Stores are guarded per element; four consecutive n of a row go out as one 8-byte store where
//    the address allows.
#pragma once
#include "gemm_mfma.hpp"
#include "gemm_mfma16.hpp"

namespace axonn {

struct EdgeCfg {
    static constexpr int BM = 128, BN = 128, BK = 128, NT = 256;
    static constexpr int PIECES = 128 * BK / 8 / NT;   // 16-byte pieces per thread, operand and K-step
    static constexpr int KC_ROW = 272;    // bytes per LDS row of a K-contiguous operand (128 k + pad)
    static constexpr int MN_ROW = 288;    // bytes per LDS k-row of an MN-contiguous operand (128 rows + pad)
    static constexpr int REGION = BK * MN_ROW;   // per operand; >= 128 * KC_ROW
    static_assert(REGION >= 128 * KC_ROW, "either layout fits a region");
    static constexpr int LDS_BYTES = 2 * REGION;
};

// Eight consecutive elements starting at p, of which the first `nvalid` (0..8) exist; the rest read as 0.
// The common cases, a whole aligned piece and no piece at all, contain no use of a loaded value and
// hence no wait: the vector loads of all pieces of a K-step are in flight together.  (Written as one
// element-wise path for everything but the whole piece, the waits inside it serialised the pieces of
// every wave that had an absent piece: an edge strip with a single valid row took twice as long as
// one with 128.)
__device__ __forceinline__ u32x4 edge_load8(const uint16_t* p, int nvalid) {
    u32x4 v{0u, 0u, 0u, 0u};
    if (nvalid == 8 && (reinterpret_cast<uintptr_t>(p) & 15) == 0) {
        v = *reinterpret_cast<const u32x4*>(p);
    } else if (nvalid > 0) {
        uint32_t e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) e[i] = i < nvalid ? (uint32_t)p[i] : 0u;
        v = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
    }
    return v;
}

// One operand's share of a thread in the staging of a K-step: PIECES 16-byte pieces.  Thread t
// takes the same 8 elements (t%16) along the contiguous dimension in 16-row steps:
//   K-contiguous  P[row * ld + k]: piece j covers row t/16 + 16 j, k = 8 (t%16) .. +7
//   MN-contiguous P[k * ld + row]: piece j covers k-row t/16 + 16 j, rows 8 (t%16) .. +7
template <bool KC>
struct EdgeOperand {
    static constexpr int NP = EdgeCfg::PIECES;
    const uint16_t* ptr0;   // first element of piece 0 at k0 = 0 (never dereferenced where nothing is valid)
    int64_t ld16;           // 16 rows (KC) or 16 k-rows (MN) on, in elements
    int64_t rows_left;      // KC: rows of the block from this thread's first row on; MN: unused
    int first;              // t/16: first row (KC) or k-row (MN) of the thread
    int kofs;               // KC: k of the pieces inside a K-step; MN: unused
    int valid;              // MN: how many of the 8 rows exist (the same for every piece); KC: unused
    uint32_t lds0;          // byte offset of piece 0 inside the operand's LDS region

    __device__ __forceinline__ void init(const uint16_t* P, int64_t row0, int64_t rows, int64_t ld, int t) {
        first = t >> 4;
        const int c = t & 15;
        ld16 = 16 * ld;
        if constexpr (KC) {
            ptr0 = P + (row0 + first) * ld + c * 8;
            rows_left = rows - (row0 + first);
            kofs = c * 8;
            valid = 0;
            lds0 = first * EdgeCfg::KC_ROW + c * 16;
        } else {
            const int64_t left = rows - (row0 + c * 8);
            ptr0 = P + first * ld + row0 + c * 8;
            rows_left = 0;
            kofs = 0;
            valid = left >= 8 ? 8 : left > 0 ? (int)left : 0;
            lds0 = first * EdgeCfg::MN_ROW + c * 16;
        }
    }
    __device__ __forceinline__ uint32_t lds(int j) const { return lds0 + j * 16 * (KC ? EdgeCfg::KC_ROW : EdgeCfg::MN_ROW); }
    // the piece j of the K-step starting at k0
    __device__ __forceinline__ u32x4 fetch(int j, int64_t k0, int64_t K) const {
        if constexpr (KC) {
            const int64_t left = K - (k0 + kofs);
            const int nvalid = 16 * j >= rows_left ? 0 : left >= 8 ? 8 : left > 0 ? (int)left : 0;
            return edge_load8(ptr0 + j * ld16 + k0, nvalid);
        } else {
            const int nvalid = k0 + first + 16 * j < K ? valid : 0;
            return edge_load8(ptr0 + (k0 / 16 + j) * ld16, nvalid);
        }
    }
};

// MFMA fragment of the 16-row block starting at row `r0` of an operand's LDS region, for the 32 k
// starting at `ks` inside the K-step: lane l gets row r0 + l%16, k = ks + 8 (l/16) .. +7.
template <bool KC>
__device__ __forceinline__ bf16x8 edge_fragment(const uint8_t* region, int r0, int ks, int lane) {
    if constexpr (KC) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(region + (r0 + (lane & 15)) * EdgeCfg::KC_ROW +
                                                                          ks * 2 + (lane >> 4) * 16));
    } else {
        // transposing read: the 16 lanes of group g = l/16 address a 4 (k) x 16 (rows) block, lane s of
        // the group k-row ks + 8g + s/4 and rows 4 (s%4) .. +3, and receive row s, four consecutive k
        typedef short i16x4 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
        const int s = lane & 15, g = lane >> 4;
        const uint8_t* p = region + (ks + 8 * g + (s >> 2)) * EdgeCfg::MN_ROW + (r0 + 4 * (s & 3)) * 2;
        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p));
        const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p + 4 * EdgeCfg::MN_ROW));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
}

// The block of the product that starts at A, B, C (already offset by the caller) and is M x N:
// workgroup (blockIdx.x % tiles_n, blockIdx.x / tiles_n) owns one 128 x 128 tile of it.
template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(256, 2) void gemm_edge_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                                        uint16_t* __restrict__ C, int64_t M, int64_t N, int64_t K,
                                                        int64_t lda, int64_t ldb, int64_t ldc, int tiles_n) {
    using Cfg = EdgeCfg;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];   // Cfg::LDS_BYTES
    uint8_t* const sa = smem;
    uint8_t* const sb = smem + Cfg::REGION;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * Cfg::BM, n0 = (int64_t)(blockIdx.x % tiles_n) * Cfg::BN;

    EdgeOperand<A_KC> oa;
    EdgeOperand<B_KC> ob;
    oa.init(A, m0, M, lda, t);
    ob.init(B, n0, N, ldb, t);

    f32x4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr int NP = Cfg::PIECES;
    u32x4 ra[NP], rb[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        ra[j] = oa.fetch(j, 0, K);
        rb[j] = ob.fetch(j, 0, K);
    }
    for (int64_t k0 = 0; k0 < K; k0 += Cfg::BK) {
        __syncthreads();   // the previous step's fragments have been read
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            *reinterpret_cast<u32x4*>(sa + oa.lds(j)) = ra[j];
            *reinterpret_cast<u32x4*>(sb + ob.lds(j)) = rb[j];
        }
        __syncthreads();
        if (k0 + Cfg::BK < K) {
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                ra[j] = oa.fetch(j, k0 + Cfg::BK, K);
                rb[j] = ob.fetch(j, k0 + Cfg::BK, K);
            }
        }
#pragma unroll
        for (int ks = 0; ks < Cfg::BK; ks += 32) {
            if (k0 + ks >= K) break;   // the rest of the step is zeros (uniform: no barrier inside)
            bf16x8 fa[4], fb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                fa[i] = edge_fragment<A_KC>(sa, wm * 64 + i * 16, ks, lane);
                fb[i] = edge_fragment<B_KC>(sb, wn * 64 + i * 16, ks, lane);
            }
            // mfma(Bfrag, Afrag): lane l then holds C[m = 16 i + l%16][n = 16 j + 4 (l/16) + e], e = 0..3
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + wm * 64 + i * 16 + (lane & 15);
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + wn * 64 + j * 16 + 4 * (lane >> 4);
            if (n >= N) continue;
            uint16_t* pc = C + m * ldc + n;
            const uint32_t lo = pack2_bf16(acc[i][j][0], acc[i][j][1]), hi = pack2_bf16(acc[i][j][2], acc[i][j][3]);
            if (n + 4 <= N && (reinterpret_cast<uintptr_t>(pc) & 7) == 0) {
                *reinterpret_cast<u32x2*>(pc) = u32x2{lo, hi};
            } else {
                pc[0] = (uint16_t)(lo & 0xFFFFu);
                if (n + 1 < N) pc[1] = (uint16_t)(lo >> 16);
                if (n + 2 < N) pc[2] = (uint16_t)(hi & 0xFFFFu);
                if (n + 3 < N) pc[3] = (uint16_t)(hi >> 16);
            }
        }
    }
}

}  // namespace axonn
