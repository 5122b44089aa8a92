// bf16 x bf16 -> fp32 -> bf16 GEMM tile kernels for gfx950 (CDNA4), one output tile per workgroup.
//
// C[M,N] = sum_k a(i,k) b(k,j)   (the local matrix multiply of Algorithm 1 lines 3, 11, 13)
//
// Design, in the order data moves:
//  * Each operand is either "K-contiguous" in global memory (A of NN/NT, B of NT) or
//    "MN-contiguous" (A of TN, B of NN/TN).  Whatever it is in global memory, the tile lands
//    in LDS in ONE canonical form: row r = the m (or n) index, 64 consecutive k as 128 bytes,
//    split into eight 16-byte chunks whose position inside the row is XOR-swizzled with
//    (r ^ r>>3) & 7.  A K-contiguous operand is copied chunk by chunk; an MN-contiguous one is
//    read as 8x8 element blocks (eight 16-byte loads along m for eight consecutive k) and
//    transposed in registers before the store.  The main loop is therefore identical for NN,
//    NT and TN.
//  * The matrix instruction is v_mfma_f32_32x32x16_bf16: lane l supplies, for row l%32, the
//    eight k values 8*(l/32)..+7 -- exactly one swizzled 16-byte LDS chunk (ds_read_b128).
//  * The products are issued as mfma(Bfrag, Afrag): the 32x32 result block then holds, in lane
//    l, column m = l%32 and FOUR CONSECUTIVE n per accumulator quad, so the epilogue can pack
//    4 bf16 into one 8-byte LDS store, transpose the tile through LDS and write C with
//    16-byte, fully coalesced global stores.
//  * LDS is double buffered: global loads for K-step t+1 are issued before the MFMAs of step
//    t and written to the other buffer afterwards; one barrier per K-step.
//  * Workgroup ids are remapped so that each of the 8 XCDs (which receive consecutive ids
//    round-robin and have private L2s) works on a compact patch of output tiles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace axonn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;          // k extent of one LDS stage
constexpr int ROW_BYTES = 128;  // BK bf16

__device__ __forceinline__ uint32_t swz(uint32_t row) { return (row ^ (row >> 3)) & 7u; }

// fp32 -> bf16 bits, round to nearest even (finite inputs; overflow rounds to inf).
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
}

// ------------------------------------------------------------------------------------------
// Global -> register -> LDS staging of one operand tile (ROWS x 64 k).
// Every global address is (wave-uniform base) + (32-bit per-thread byte offset that never
// changes), so the loop advances only scalar registers.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ u32x4 ld_global_16(const uint8_t* uniform_base, uint32_t voff) {
    return *reinterpret_cast<const u32x4*>(uniform_base + voff);
}

template <int ROWS, int NT, bool KCONTIG>
struct TileLoader;

// K-contiguous: P[row * ld + k].  Thread t handles chunks t, t+NT, ...; chunk = (row, ck):
// eight consecutive lanes cover the 128 contiguous bytes of one row.
template <int ROWS, int NT>
struct TileLoader<ROWS, NT, true> {
    static constexpr int CH = (ROWS * 8) / NT;
    static constexpr int NLOADS = CH, NSTORES = CH;
    static_assert(CH >= 1 && (ROWS * 8) % NT == 0, "tile/threads mismatch");
    // Pass c handles rows row + c*NT/8.  With NT a multiple of 256 that adds a multiple of 4 to
    // row>>3, i.e. flips bit 2 of swz(row) for odd multiples and nothing else: an XOR constant.
    static_assert(NT % 256 == 0, "swizzle of later passes assumes NT/8 is a multiple of 32");
    __device__ __forceinline__ static constexpr uint32_t pass_xor(int c) { return ((c * (NT / 64)) & 7) << 4; }
    u32x4 reg[CH];
    uint32_t voff, lds_off;
    uint32_t pass_bytes;  // uniform: global distance between the rows of two passes

    __device__ __forceinline__ void init(int t, uint32_t ld_bytes) {
        const uint32_t row = t >> 3, ck = t & 7;
        voff = row * ld_bytes + ck * 16;
        pass_bytes = (NT / 8) * ld_bytes;
        lds_off = row * ROW_BYTES + ((ck ^ swz(row)) << 4);
    }
    __device__ __forceinline__ void load(const uint8_t* tile) {
#pragma unroll
        for (int c = 0; c < CH; ++c) reg[c] = ld_global_16(tile + (size_t)c * pass_bytes, voff);
    }
    __device__ __forceinline__ void store(uint8_t* lds) const {
#pragma unroll
        for (int c = 0; c < CH; ++c)
            *reinterpret_cast<u32x4*>(lds + (lds_off ^ pass_xor(c)) + c * (NT / 8) * ROW_BYTES) = reg[c];
    }
    __device__ __forceinline__ static size_t kstep_bytes(uint32_t) { return BK * 2; }
};

// MN-contiguous: P[k * ld + row].  Thread t handles 8x8 element blocks; block = (mb, kb):
// lanes 0..7 take 8 consecutive m-blocks (128 contiguous bytes for each k), lane/8 picks kb.
template <int ROWS, int NT>
struct TileLoader<ROWS, NT, false> {
    static constexpr int BLOCKS = ROWS;  // (ROWS/8) m-blocks x 8 k-blocks
    static constexpr int NB = (BLOCKS + NT - 1) / NT;
    static constexpr bool PARTIAL = (BLOCKS % NT) != 0;  // only the first BLOCKS threads work
    static constexpr int NLOADS = 8 * NB, NSTORES = 8 * NB;
    static_assert(BLOCKS % 64 == 0, "whole waves only");
    static_assert(!PARTIAL || NB == 1, "partial pass only when there is a single pass");
    u32x4 reg[NB][8];
    uint32_t voff, lds_off, ld_b;
    bool active;

    __device__ __forceinline__ void init(int t, uint32_t ld_bytes) {
        const uint32_t mb = (t & 7) | ((t >> 6) << 3), kb = (t >> 3) & 7;
        ld_b = ld_bytes;
        voff = kb * 8 * ld_bytes + mb * 16;
        active = !PARTIAL || t < BLOCKS;
        // row = mb*8 + i: swz(row) = (i ^ mb) & 7, so store i goes to chunk kb ^ ((i ^ mb) & 7)
        lds_off = mb * 8 * ROW_BYTES;
        kb_ = kb;
        mb_ = mb;
    }
    __device__ __forceinline__ void load(const uint8_t* tile) {
        if (!active) return;  // wave-uniform
#pragma unroll
        for (int c = 0; c < NB; ++c)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                reg[c][j] = ld_global_16(tile + (size_t)j * ld_b + (size_t)c * (NT / 64) * 128, voff);
    }
    __device__ __forceinline__ void store(uint8_t* lds) const {
        if (!active) return;
#pragma unroll
        for (int c = 0; c < NB; ++c) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                // output row i of the block: element i of each of the eight k-rows
                u32x4 o;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t x = reg[c][2 * q][i >> 1], y = reg[c][2 * q + 1][i >> 1];
                    o[q] = (i & 1) ? ((x >> 16) | (y & 0xFFFF0000u)) : ((x & 0xFFFFu) | (y << 16));
                }
                // pass c covers m-blocks mb + c*NT/8 (a multiple of 8 further: same swizzle)
                const uint32_t sw = (kb_ ^ i ^ mb_) & 7;
                *reinterpret_cast<u32x4*>(lds + lds_off + (c * (NT / 8) * 8 + i) * ROW_BYTES + (sw << 4)) = o;
            }
        }
    }
    __device__ __forceinline__ static size_t kstep_bytes(uint32_t ld_bytes) { return (size_t)BK * ld_bytes; }
    uint32_t kb_, mb_;
};

// A run of scheduling groups: NM MFMAs with NR LDS reads, NV global loads and NW LDS writes
// spread evenly between them (compile-time recursion: the builtin wants literal counts).
template <int MASK, int N>
__device__ __forceinline__ void sched_group() {
    if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(MASK, N, 0);
}
template <int NM, int NR, int NV, int NW, int I = 0>
__device__ __forceinline__ void interleave_hint() {
    if constexpr (I < NM) {
        sched_group<0x008, 1>();                                          // one MFMA
        sched_group<0x020, ((I + 1) * NV) / NM - (I * NV) / NM>();        // global loads
        sched_group<0x100, ((I + 1) * NR) / NM - (I * NR) / NM>();        // LDS reads
        sched_group<0x200, ((I + 1) * NW) / NM - (I * NW) / NM>();        // LDS writes
        interleave_hint<NM, NR, NV, NW, I + 1>();
    }
}

// ------------------------------------------------------------------------------------------
// The tile kernel.
//   BM x BN output tile, WM x WN waves, each wave a (BM/WM) x (BN/WN) sub-tile of 32x32 blocks.
//   Requires M % BM == 0, N % BN == 0, K % 64 == 0 (checked on the host).
// ------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN>
struct TileCfg {
    static constexpr int NT = WM * WN * 64;
    static constexpr int TM = BM / WM, TN = BN / WN;
    static constexpr int MI = TM / 32, NI = TN / 32;
    static constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
    static constexpr int EPI_BYTES = BM * BN * 2;
    static constexpr int LDS_BYTES = (2 * STAGE_BYTES > EPI_BYTES) ? 2 * STAGE_BYTES : EPI_BYTES;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be whole 32x32 blocks");
};

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(WM* WN * 64) void gemm_tile_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
    int M, int N, int K, int tiles_m, int tiles_n, int group_m) {
    using Cfg = TileCfg<BM, BN, WM, WN>;
    constexpr int NT = Cfg::NT, TM = Cfg::TM, TN = Cfg::TN, MI = Cfg::MI, NI = Cfg::NI;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- workgroup -> output tile: XCD-contiguous, then grouped along m --------------------
    int pid = blockIdx.x;
    const int nwg = gridDim.x;
    if ((nwg & 7) == 0) pid = (pid & 7) * (nwg >> 3) + (pid >> 3);
    const int group_sz = group_m * tiles_n;
    const int group = pid / group_sz;
    const int first_m = group * group_m;
    const int gm = min(tiles_m - first_m, group_m);
    const int in_group = pid - group * group_sz;
    const int tile_m = first_m + in_group % gm;
    const int tile_n = in_group / gm;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

    const uint32_t lda_b = 2u * (uint32_t)(A_KC ? K : M);  // leading dimensions in bytes
    const uint32_t ldb_b = 2u * (uint32_t)(B_KC ? K : N);
    const uint8_t* pa = reinterpret_cast<const uint8_t*>(A) + (A_KC ? (size_t)m0 * lda_b : (size_t)m0 * 2);
    const uint8_t* pb = reinterpret_cast<const uint8_t*>(B) + (B_KC ? (size_t)n0 * ldb_b : (size_t)n0 * 2);

    using LoaderA = TileLoader<BM, NT, A_KC>;
    using LoaderB = TileLoader<BN, NT, B_KC>;
    LoaderA la;
    LoaderB lb;
    la.init(t, lda_b);
    lb.init(t, ldb_b);
    constexpr int NLOADS = LoaderA::NLOADS + LoaderB::NLOADS;
    constexpr int NSTORES = LoaderA::NSTORES + LoaderB::NSTORES;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // per-lane fragment addresses inside a stage (bytes), for k-substep 0; substep s flips
    // chunk bits 1..2, which is XOR (s << 5) on the byte offset.
    const uint32_t half = lane >> 5, r32 = lane & 31;
    uint32_t a_off[MI], b_off[NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const uint32_t row = wm * TM + i * 32 + r32;
        a_off[i] = row * ROW_BYTES + ((half ^ swz(row)) << 4);
    }
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const uint32_t row = wn * TN + j * 32 + r32;
        b_off[j] = BM * ROW_BYTES + row * ROW_BYTES + ((half ^ swz(row)) << 4);
    }

    // Register double buffer of MFMA operand fragments: the LDS reads of k-substep s+1 are
    // issued before the MFMAs of substep s, and the last substep of a K-step is issued AFTER
    // the barrier together with the first reads of the next stage, so neither LDS latency
    // nor the barrier leaves the matrix pipe without queued work.
    bf16x8 af[2][MI], bf[2][NI];
    auto read_frags = [&](const uint8_t* stage, int s, int buf) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
            af[buf][i] = *reinterpret_cast<const bf16x8*>(stage + (a_off[i] ^ (s << 5)));
#pragma unroll
        for (int j = 0; j < NI; ++j)
            bf[buf][j] = *reinterpret_cast<const bf16x8*>(stage + (b_off[j] ^ (s << 5)));
    };
    auto mfma_block = [&](int buf) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[buf][j], af[buf][i], acc[i][j], 0, 0, 0);
    };
    constexpr int NM = MI * NI, NR = MI + NI;

    const int KT = K / BK;
    la.load(pa);
    lb.load(pb);
    la.store(smem);
    lb.store(smem + BM * ROW_BYTES);
    __syncthreads();
    read_frags(smem, 0, 0);

    for (int kt = 0; kt + 1 < KT; ++kt) {
        const uint8_t* cur = smem + (kt & 1) * Cfg::STAGE_BYTES;
        uint8_t* nxt = smem + ((kt + 1) & 1) * Cfg::STAGE_BYTES;
        pa += LoaderA::kstep_bytes(lda_b);
        pb += LoaderB::kstep_bytes(ldb_b);
        // substep 0: global loads of the next K-step ride along
        la.load(pa);
        lb.load(pb);
        read_frags(cur, 1, 1);
        mfma_block(0);
        interleave_hint<NM, NR, NLOADS, 0>();
        __builtin_amdgcn_sched_barrier(0);
        // substep 1
        read_frags(cur, 2, 0);
        mfma_block(1);
        interleave_hint<NM, NR, 0, 0>();
        __builtin_amdgcn_sched_barrier(0);  // nothing of the LDS refill may start before here
        // substep 2: the loaded tile goes to the other LDS stage between the MFMAs
        read_frags(cur, 3, 1);
        mfma_block(0);
        la.store(nxt);
        lb.store(nxt + BM * ROW_BYTES);
        // (LDS reads first: a write may not be scheduled above a read it could alias)
        interleave_hint<NM / 2, NR, 0, 0>();
        interleave_hint<NM - NM / 2, 0, 0, NSTORES>();
        __syncthreads();
        // substep 3 runs after the barrier, next to the first reads of the next stage
        read_frags(nxt, 0, 0);
        mfma_block(1);
        interleave_hint<NM, NR, 0, 0>();
    }
    {
        const uint8_t* cur = smem + ((KT - 1) & 1) * Cfg::STAGE_BYTES;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            read_frags(cur, s + 1, (s + 1) & 1);
            mfma_block(s & 1);
            interleave_hint<NM, NR, 0, 0>();
        }
        mfma_block(1);
        __syncthreads();  // every wave is done reading LDS before the epilogue reuses it
    }

    // ---- epilogue: fp32 -> bf16, transpose through this wave's private LDS region ----------
    // acc[i][j][4g + e] = C[m = i*32 + l%32][n = j*32 + 8g + 4*(l/32) + e]
    constexpr int CPR = TN / 8;  // 16-byte chunks per row of the wave tile
    constexpr uint32_t CMASK = (CPR >= 16 ? 16 : CPR) - 1;
    uint8_t* epi = smem + wave * (TM * TN * 2);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t row = i * 32 + r32;
                const uint32_t chunk = j * 4 + g;
                u32x2 v;
                v[0] = pack2_bf16(acc[i][j][4 * g + 0], acc[i][j][4 * g + 1]);
                v[1] = pack2_bf16(acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
                *reinterpret_cast<u32x2*>(epi + row * (TN * 2) + ((chunk ^ (row & CMASK)) << 4) + half * 8) = v;
                if (g == 3) __builtin_amdgcn_sched_barrier(0);  // keep the conversion block by block
            }
    __syncthreads();
    uint16_t* pc = C + (m0 + wm * TM) * (int64_t)N + n0 + wn * TN;
#pragma unroll
    for (int it = 0; it < (TM * CPR) / 64; ++it) {
        const uint32_t idx = it * 64 + lane;
        const uint32_t row = idx / CPR, ch = idx % CPR;
        const u32x4 v = *reinterpret_cast<const u32x4*>(epi + row * (TN * 2) + ((ch ^ (row & CMASK)) << 4));
        *reinterpret_cast<u32x4*>(pc + (int64_t)row * N + ch * 8) = v;
    }
}

}  // namespace axonn
