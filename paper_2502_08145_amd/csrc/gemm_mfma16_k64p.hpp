// The 64-k-stage tile kernel as ONE RESIDENT WORKGROUP PER COMPUTE UNIT that walks a list of output
// tiles (no split-K).  Same operand staging, fragments, MFMA order and LDS buffers as
// gemm_tile_kernel_k64 (eight waves, 2 x 4); what changes is what happens between two tiles.
//
// Measured with per-workgroup time stamps on the one-tile-per-workgroup kernel (4096 x 16384 x 2048, TN,
// four rounds of 256 tiles, 53.7 us per round): 46.2 us of K loop, and around it 7.5 us in which the
// matrix pipes of the compute unit idle: 2.0 us from a workgroup's last instruction to its successor's
// first (its stores drain, the next workgroup is dispatched), 3.5 us until the successor's first
// panels have landed (1.3 us of that to get the thirty-two loads of a wave issued at all: every
// compute unit of the chip starts its burst at the same moment), and 2 us of epilogue.
//
// Here the load stream never stops: the direct loads that a workgroup issues two iterations ahead
// simply move on to the next tile's panels while the last two iterations of the running tile are
// multiplied, so a tile's first panels are in LDS when its predecessor's last MFMA is issued; there is
// no dispatch between tiles and nothing drains.  C leaves block row by block row during the tile's
// last sub-step (staged through the 32 KB of LDS that the two 64 KB buffers leave free, so the
// buffers can already hold the next tile), and the accumulators are cleared row by row behind it.
// The one thing that cannot be avoided: loads and stores share one in-order counter on this chip,
// so the first barrier of the next tile (vmcnt(0): "my share of the panels has landed") also waits
// for the C stores to be acknowledged.
//
// Workgroup b of a grid of G takes the tiles b, b + G, b + 2G, ... of the XCD-aware tile sequence
// (map_workgroup): the tiles that run side by side are the same as with one workgroup per tile, and
// so is what the L2s see.
#pragma once
#include "gemm_mfma16_k64.hpp"

namespace axonn {

struct TileCfgK64P {
    static constexpr int EPI_OFFSET = TileCfgK64::LDS_BYTES;        // staging area behind the two buffers
    static constexpr int EPI_BYTES = 8 * 16 * 64 * 2;               // eight waves x one block row of 16 x 64 bf16
    static constexpr int LDS_BYTES = EPI_OFFSET + EPI_BYTES;        // 144 KB
    static constexpr int MAX_WORKGROUPS = 256;                      // one per compute unit
};

// Requires M % 256 == 0, N % 256 == 0, K % 64 == 0, K >= 128; gridDim.x <= tiles, and a multiple of 8
// whenever the number of tiles is one (keeps a workgroup's tiles on the XCD that map_workgroup means them for).
template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(512) void gemm_tile_kernel_k64p(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
    int K, int lda, int ldb, int ldc, int tiles_m, int tiles_n, int group_m, SplitK sk) {
    using Cfg = TileCfgK64;
    constexpr int WN = 4, BM = Cfg::BM, BN = Cfg::BN, NW = 8;
    constexpr int TM = BM / 2, TN = BN / WN, MI = TM / 16, NI = TN / 16, NM = MI * NI;
    constexpr uint32_t BUF = Cfg::BUF_BYTES, REGION_B = Cfg::A_BYTES;
    constexpr int QL = 32 / NW;
    constexpr int NLD = 2 * QL, NRD = MI + NI;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int total = tiles_m * tiles_n;
    const int stride = (int)gridDim.x;

    int pid = (int)blockIdx.x;
    TileWork work = map_workgroup<false, true>(pid, total, K, tiles_m, tiles_n, group_m, sk);

    using OpA = typename std::conditional<A_KC, OperandK64KContig<BM, 0, NW>, OperandK64MNContig<BM, 0, NW, MI / 2>>::type;
    using OpB = typename std::conditional<B_KC, OperandK64KContig<BN, REGION_B, NW>, OperandK64MNContig<BN, REGION_B, NW, NI / 2>>::type;
    static_assert(OpA::QL == QL && OpB::QL == QL, "loads per wave");
    const uint32_t lds0 = lds_address(smem);
    OpA opa;
    OpB opb;
    opa.init(A, (int64_t)work.tile_m * BM, 2u * (uint32_t)lda, lane, wave, lds0, wm * TM);
    opb.init(B, (int64_t)work.tile_n * BN, 2u * (uint32_t)ldb, lane, wave, lds0, wn * TN);
    auto issue = [&](auto x_c, uint32_t buf) __attribute__((always_inline)) {
        constexpr int X = decltype(x_c)::value;
        if constexpr (X < QL)
            opa.template issue<X>(buf);
        else
            opb.template issue<X - QL>(buf);
    };
    auto advance_window = [&]() __attribute__((always_inline)) {
        opa.advance();
        opb.advance();
    };

    f32x4 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    typename OpA::Frag fa[2][MI];
    typename OpB::Frag fb[2][NI];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[u][i].clear();
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[u][j].clear();
    }

#define AXONN_FENCE() __builtin_amdgcn_sched_barrier(0)
    auto mfma_range = [&](auto s_c, auto lo_c, auto hi_c) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value, LO = decltype(lo_c)::value, HI = decltype(hi_c)::value;
        static_for<HI - LO>([&](auto d) __attribute__((always_inline)) {
            // block rows in order, the blocks of a row back and forth: from one MFMA to the next exactly one
            // operand changes (0.3-0.5 % on the benchmark step in alternating runs: less toggling on the
            // operand buses of a power-limited chip)
            constexpr int I = (LO + decltype(d)::value) / NI, J0 = (LO + decltype(d)::value) % NI;
            constexpr int J = (I & 1) ? NI - 1 - J0 : J0;
            acc[I][J] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[S][J].get(), fa[S][I].get(), acc[I][J], 0, 0, 0);
        });
    };
    auto wait_fragments = [&](auto s_c) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value;
        static_for<MI / 4>([&](auto d) __attribute__((always_inline)) { tie_to_lds_wait<4>(&fa[S][4 * decltype(d)::value]); });
        static_for<NI / 4>([&](auto d) __attribute__((always_inline)) { tie_to_lds_wait<4>(&fb[S][4 * decltype(d)::value]); });
    };
    // cluster Q of NCX: its share of the fragment reads of a sub-step into register buffer S (A blocks,
    // then B), and of the direct loads of an iteration
    constexpr int NC = (!A_KC && !B_KC) ? 6 : 4;
    constexpr int PB = NM / 8;
    auto read_cluster = [&](auto q_c, auto ncx_c, auto s_c, const typename OpA::Cursor& ca, const typename OpB::Cursor& cb) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value, NCX = decltype(ncx_c)::value, S = decltype(s_c)::value;
        constexpr int RF = Q * NRD / NCX, RL = (Q + 1) * NRD / NCX;
        static_for<RL - RF>([&](auto d) __attribute__((always_inline)) {
            constexpr int X = RF + decltype(d)::value;
            if constexpr (X < MI)
                opa.template read<X>(fa[S][X], ca);
            else
                opb.template read<X - MI>(fb[S][X - MI], cb);
        });
    };
    auto load_cluster = [&](auto q_c, auto ncx_c, uint32_t buf) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value, NCX = decltype(ncx_c)::value;
        constexpr int LF = Q * NLD / NCX, LL = (Q + 1) * NLD / NCX;
        static_for<LL - LF>([&](auto d) __attribute__((always_inline)) { issue(Int<LF + decltype(d)::value>{}, buf); });
    };

    // ---- prologue: iterations 0 and 1 of the first tile into buffers 0 and 1 -------------------------
    static_for<NLD>([&](auto x) __attribute__((always_inline)) { issue(x, 0u); });
    advance_window();
    static_for<NLD>([&](auto x) __attribute__((always_inline)) { issue(x, BUF); });
    advance_window();
    wait_vmcnt<NLD>();
    __builtin_amdgcn_s_barrier();
    AXONN_FENCE();
    {
        const typename OpA::Cursor ca = opa.template cursor<0>(0u);
        const typename OpB::Cursor cb = opb.template cursor<0>(0u);
        static_for<NC>([&](auto q_c) __attribute__((always_inline)) { read_cluster(q_c, Int<NC>{}, Int<0>{}, ca, cb); });
    }

    uint32_t cur = 0;
    // One sub-step S of the running iteration (see gemm_tile_kernel_k64): fragments of the following
    // sub-step are read; in sub-step 1, after the barrier, the loads of the iteration after next go
    // out into the running buffer.  Every iteration reads and loads: what follows a tile's last
    // iterations is the next tile (or, behind the last tile, panels that nobody multiplies).
    auto substep = [&](auto s_c) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value;
        constexpr int R = 3 * NM / 4 - PB;
        wait_fragments(s_c);
        AXONN_FENCE();
        mfma_range(s_c, Int<0>{}, Int<PB>{});
        AXONN_FENCE();
        typename OpA::Cursor ca = opa.template cursor<1 - S>(S == 1 ? cur ^ BUF : cur);
        typename OpB::Cursor cb = opb.template cursor<1 - S>(S == 1 ? cur ^ BUF : cur);
        if constexpr (S == 1) {
            wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            AXONN_FENCE();
        }
        static_for<NC>([&](auto q_c) __attribute__((always_inline)) {
            constexpr int Q = decltype(q_c)::value;
            read_cluster(q_c, Int<NC>{}, Int<1 - S>{}, ca, cb);
            if constexpr (S == 1) load_cluster(q_c, Int<NC>{}, cur);
            AXONN_FENCE();
            if constexpr (Q < NC - 1)
                mfma_range(s_c, Int<PB + Q * R / (NC - 1)>{}, Int<PB + (Q + 1) * R / (NC - 1)>{});
            else
                mfma_range(s_c, Int<PB + R>{}, Int<NM>{});
            AXONN_FENCE();
        });
        if constexpr (S == 1) {
            advance_window();
            cur ^= BUF;
        }
    };
    // The last sub-step of a tile: the same reads, loads and barrier, but the MFMAs go block row by block
    // row, and a finished block row is converted, staged (this wave's 2 KB behind the buffers), stored
    // and cleared while the next rows are multiplied.  The reads and loads are dealt out over the rows
    // 1 .. MI-2.
    auto last_substep = [&](uint16_t* pc) __attribute__((always_inline)) {
        constexpr int NCE = MI - 2;
        wait_fragments(Int<1>{});
        AXONN_FENCE();
        mfma_range(Int<1>{}, Int<0>{}, Int<NI>{});
        AXONN_FENCE();
        typename OpA::Cursor ca = opa.template cursor<0>(cur ^ BUF);
        typename OpB::Cursor cb = opb.template cursor<0>(cur ^ BUF);
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        AXONN_FENCE();
        uint8_t* const epi = smem + TileCfgK64P::EPI_OFFSET + wave * (16 * TN * 2);
        // the lane number through an opaque move: everything the epilogue derives from it (staging and
        // store addresses) is then computed here, not hoisted out of the tile loop and kept in registers
        // across the K loop, where there are none to spare
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        static_for<MI - 1>([&](auto d) __attribute__((always_inline)) {
            constexpr int I = decltype(d)::value + 1;
            if constexpr (I - 1 < NCE) {
                read_cluster(Int<I - 1>{}, Int<NCE>{}, Int<0>{}, ca, cb);
                load_cluster(Int<I - 1>{}, Int<NCE>{}, cur);
                AXONN_FENCE();
            }
            mfma_range(Int<1>{}, Int<I * NI>{}, Int<(I + 1) * NI>{});
            AXONN_FENCE();
            store_block_row16<TN, NI>(acc[I - 1], epi, pc + (int64_t)((I - 1) * 16) * ldc, ldc, lane_e);
#pragma unroll
            for (int j = 0; j < NI; ++j) acc[I - 1][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            AXONN_FENCE();
        });
        store_block_row16<TN, NI>(acc[MI - 1], epi, pc + (int64_t)((MI - 1) * 16) * ldc, ldc, lane_e);
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[MI - 1][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        AXONN_FENCE();
        advance_window();
        cur ^= BUF;
    };

    const int KI = K / Cfg::KS;   // at least 2
    for (;;) {
        const int next = pid + stride;
        const bool has_next = next < total;
        // the tile whose panels the loads turn to two iterations before this one ends: the next tile,
        // or, behind the last one, this tile once more (valid addresses, nobody multiplies them)
        const TileWork nw = has_next ? map_workgroup<false, true>(next, total, K, tiles_m, tiles_n, group_m, sk) : work;
        for (int it = 0; it < KI - 1; ++it) {
            if (it == KI - 2) {
                opa.retarget(A, (int64_t)nw.tile_m * BM, 2u * (uint32_t)lda, wave, 2u * (uint32_t)K);
                opb.retarget(B, (int64_t)nw.tile_n * BN, 2u * (uint32_t)ldb, wave, 2u * (uint32_t)K);
            }
            substep(Int<0>{});
            substep(Int<1>{});
        }
        substep(Int<0>{});
        last_substep(C + ((int64_t)work.tile_m * BM + wm * TM) * (int64_t)ldc + (int64_t)work.tile_n * BN + wn * TN);
        if (!has_next) break;
        pid = next;
        work = nw;
    }
#undef AXONN_FENCE
}

}  // namespace axonn
