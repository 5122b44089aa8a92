// The NT product (both operands K-contiguous in memory: A[m][k], B[n][k]) with LDS stages of 64 k.
//
// Why a kernel of its own.  In gemm_tile_kernel16 a K-contiguous operand is staged 32 k at a time:
// a row of a stage is 64 bytes, half a cache line, so every direct load asks the L1 for sixteen
// half lines, and the 8-wave layout reads every LDS byte three times.  With both operands
// K-contiguous the panels can instead be staged 64 k at a time:
//
//  * an LDS row is one whole 128-byte line (row r, the eight 16-byte chunks XOR-swizzled by
//    (r>>1)&7: ds_read_b128 of sixteen consecutive rows then touches every bank once), a direct
//    load fetches 8 rows x 128 B: eight full-line requests instead of sixteen half-line ones;
//  * two buffers of (256 + 256) rows x 128 B = 64 KB each; 4 waves (2 x 2), wave tile 128 x 128:
//    every LDS byte is read twice, not three times;
//  * ONE barrier per 64 k.  An iteration is two sub-steps of 32 k (64 MFMAs per wave each).  During
//    sub-step 0 of iteration i the fragments of its sub-step 1 are read; during sub-step 1, after
//    the barrier, the fragments of iteration i+1 (other buffer), and the direct loads of iteration
//    i+2 go out into the buffer that iteration i has just finished with.  At the barrier every
//    load issued so far must have landed (vmcnt(0)): those of iteration i+1, issued one iteration
//    earlier, i.e. a lead of almost two sub-steps.
//
// Fragments, MFMA order (mfma(Bfrag, Afrag)), accumulator layout, split-K exchange, epilogue and
// the XCD-aware tile order are those of gemm_tile_kernel16.
#pragma once
#include "gemm_mfma16.hpp"

namespace axonn {

struct TileCfgK64 {
    static constexpr int BM = 256, BN = 256, NW = 4, NT = 256;
    static constexpr int KS = 64;                                  // k per LDS buffer
    static constexpr int A_BYTES = BM * KS * 2, BUF_BYTES = (BM + BN) * KS * 2;
    static constexpr int LDS_BYTES = 2 * BUF_BYTES;                // 128 KB; the epilogue needs BM*BN*2 = 128 KB
    static constexpr int MIN_K = 2 * KS;                           // the prologue fills both buffers
};

// Requires M % 256 == 0, N % 256 == 0, K % 64 == 0, K >= 128 (per K range when split).
template <bool SPLITK>
__global__ __launch_bounds__(256) void gemm_tile_kernel_k64(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
    int K, int lda, int ldb, int ldc, int tiles_m, int tiles_n, int group_m, SplitK sk) {
    using Cfg = TileCfgK64;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, NW = 4, WN = 2;
    constexpr int TM = 128, TN = 128, MI = 8, NI = 8, NM = MI * NI;
    constexpr uint32_t BUF = Cfg::BUF_BYTES, REGION_B = Cfg::A_BYTES;
    constexpr int QL = 8;   // direct loads per wave, operand and iteration: 8 row groups of 8 rows
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- workgroup -> output tile and K range (as in gemm_tile_kernel) -------------------------
    int pid = blockIdx.x;
    const int nwg = gridDim.x;
    int krange = 0, ktotal = K;
    if constexpr (SPLITK) {
        const int splits = sk.splits, tiles = tiles_m * tiles_n;
        if (splits == 4 && (nwg & 7) == 0 && K >= kSplitRangePerXcdK) {
            const int x = pid & 7, q = pid >> 3, tp = tiles >> 1;
            krange = 3 - (x >> 1);
            pid = (x & 1) * tp + q;
        } else if (nwg % (8 * splits) == 0) {
            const int tp = (nwg >> 3) / splits, li = pid >> 3;
            krange = splits - 1 - li / tp;
            pid = (pid & 7) * tp + li % tp;
        } else {
            krange = splits - 1 - pid / tiles;
            pid = pid % tiles;
        }
        ktotal = K / splits;
    } else {
        if ((nwg & 7) == 0) pid = (pid & 7) * (nwg >> 3) + (pid >> 3);
    }
    const int tile_id = pid;
    const int group_sz = group_m * tiles_n;
    const int group = pid / group_sz;
    const int first_m = group * group_m;
    const int gm = min(tiles_m - first_m, group_m);
    const int in_group = pid - group * group_sz;
    const int tile_m = first_m + in_group % gm;
    const int tile_n = in_group / gm;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int64_t k0 = (int64_t)krange * ktotal;

    // ---- direct loads: this wave fetches row groups 8*wave .. 8*wave+7 of either operand ------------
    // Lane l of a load lands at (row l/8, slot l%8) of its group; slot s of row r holds chunk
    // s ^ ((r>>1)&7), and (r>>1)&7 = 4*(group&1) + l/16: one per-lane offset for the even groups and
    // one for the odd ones.
    const uint32_t lds0 = lds_address(smem);
    const uint32_t lda_b = 2u * (uint32_t)lda, ldb_b = 2u * (uint32_t)ldb;
    const uint8_t* base_a[QL];
    const uint8_t* base_b[QL];
#pragma unroll
    for (int c = 0; c < QL; ++c) {
        base_a[c] = reinterpret_cast<const uint8_t*>(A + k0) + (size_t)(m0 + 8 * (QL * wave + c)) * lda_b;
        base_b[c] = reinterpret_cast<const uint8_t*>(B + k0) + (size_t)(n0 + 8 * (QL * wave + c)) * ldb_b;
    }
    const uint32_t lds_dst_a = lds0 + (uint32_t)(QL * wave) * 1024u, lds_dst_b = lds_dst_a + REGION_B;
    uint32_t voff_a[2], voff_b[2];   // [group parity]; advance 128 bytes per iteration
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const uint32_t chunk = (uint32_t)(lane & 7) ^ (uint32_t)(4 * p + (lane >> 4));
        voff_a[p] = (uint32_t)(lane >> 3) * lda_b + (chunk << 4);
        voff_b[p] = (uint32_t)(lane >> 3) * ldb_b + (chunk << 4);
    }
    // load number X of an iteration (0..7: A groups, 8..15: B groups) into the buffer at `buf`
    auto issue = [&](auto x_c, uint32_t buf) __attribute__((always_inline)) {
        constexpr int X = decltype(x_c)::value, G = X % QL;
        if constexpr (X < QL)
            direct_load16(lds_dst_a + buf + G * 1024u, base_a[G], voff_a[G & 1]);
        else
            direct_load16(lds_dst_b + buf + G * 1024u, base_b[G], voff_b[G & 1]);
    };
    auto advance_window = [&]() __attribute__((always_inline)) {
        voff_a[0] += 2 * Cfg::KS; voff_a[1] += 2 * Cfg::KS;
        voff_b[0] += 2 * Cfg::KS; voff_b[1] += 2 * Cfg::KS;
    };

    // ---- fragment reads: lane l wants, for 16-row block I and sub-step s, row 16*I + l%16 and chunk
    // 4*s + l/16; that chunk sits in slot (4*s + l/16) ^ ((l%16)>>1).  Block I is an immediate offset
    // of I * 2048.
    const uint32_t r16 = lane & 15, quad = lane >> 4;
    uint32_t raddr_a[2], raddr_b[2];   // [sub-step]
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t slot = ((uint32_t)(4 * s) + quad) ^ (r16 >> 1);
        raddr_a[s] = lds0 + (uint32_t)(wm * TM + r16) * 128u + (slot << 4);
        raddr_b[s] = lds0 + REGION_B + (uint32_t)(wn * TN + r16) * 128u + (slot << 4);
    }

    f32x4 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    Frag128 fa[2][MI], fb[2][NI];   // [sub-step][block]; pinned registers (see lds_read128)
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
            constexpr int I = (LO + decltype(d)::value) / NI, J = (LO + decltype(d)::value) % NI;
            acc[I][J] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[S][J].get(), fa[S][I].get(), acc[I][J], 0, 0, 0);
        });
    };
    auto wait_fragments = [&](auto s_c) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value;
        tie_to_lds_wait<4>(&fa[S][0]);
        tie_to_lds_wait<4>(&fa[S][4]);
        tie_to_lds_wait<4>(&fb[S][0]);
        tie_to_lds_wait<4>(&fb[S][4]);
    };
    // cluster Q of NC: its share of the sixteen fragment reads of a sub-step into register buffer S
    // (A blocks, then B), and of the sixteen direct loads of an iteration
#ifndef AXONN_K64_NC
#define AXONN_K64_NC 4
#endif
#ifndef AXONN_K64_PB
#define AXONN_K64_PB 8
#endif
#ifndef AXONN_K64_LAST
#define AXONN_K64_LAST 47
#endif
    constexpr int NC = AXONN_K64_NC, PER = 16 / NC;
    auto read_cluster = [&](auto q_c, auto s_c, uint32_t addr_a, uint32_t addr_b) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value, S = decltype(s_c)::value;
        static_for<PER>([&](auto d) __attribute__((always_inline)) {
            constexpr int X = PER * Q + decltype(d)::value;
            if constexpr (X < MI)
                lds_read128<X * 2048>(fa[S][X].v, addr_a);
            else
                lds_read128<(X - MI) * 2048>(fb[S][X - MI].v, addr_b);
        });
    };
    auto load_cluster = [&](auto q_c, uint32_t buf) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value;
        static_for<PER>([&](auto d) __attribute__((always_inline)) { issue(Int<PER * Q + decltype(d)::value>{}, buf); });
    };

    // ---- prologue: iterations 0 and 1 into buffers 0 and 1 -----------------------------------------
    static_for<16>([&](auto x) __attribute__((always_inline)) { issue(x, 0u); });
    advance_window();
    static_for<16>([&](auto x) __attribute__((always_inline)) { issue(x, BUF); });
    advance_window();
    wait_vmcnt<16>();   // iteration 0 has landed
    __builtin_amdgcn_s_barrier();
    AXONN_FENCE();

    // `cur`: byte offset of the buffer of the running iteration
    uint32_t cur = 0;
    // One sub-step S of the running iteration.
    //   READ: fragments for the following sub-step are read (S = 0: sub-step 1 of the same buffer;
    //         S = 1: sub-step 0 of the other buffer, after the barrier).
    //   LOAD (S = 1): the iteration after next is fetched into the running buffer, after the barrier.
    auto substep = [&](auto s_c, auto read_c, auto load_c) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value;
        constexpr bool READ = decltype(read_c)::value, LOAD = decltype(load_c)::value;
        static_assert(!LOAD || (S == 1 && READ), "loads go out in sub-step 1 of an iteration that has a successor");
        constexpr int PB = AXONN_K64_PB, DP = (AXONN_K64_LAST - PB) / (NC - 1);
        wait_fragments(s_c);
        AXONN_FENCE();
        mfma_range(s_c, Int<0>{}, Int<PB>{});
        AXONN_FENCE();
        uint32_t addr_a = 0, addr_b = 0;
        if constexpr (READ) {
            if constexpr (S == 1) {
                wait_vmcnt<0>();                 // the next iteration's panels: every load of this wave ...
                __builtin_amdgcn_s_barrier();    // ... and of the others; and the running buffer is free
                AXONN_FENCE();
                addr_a = raddr_a[0] + (cur ^ BUF);
                addr_b = raddr_b[0] + (cur ^ BUF);
            } else {
                addr_a = raddr_a[1] + cur;
                addr_b = raddr_b[1] + cur;
            }
        }
        static_for<NC>([&](auto q_c) __attribute__((always_inline)) {
            constexpr int Q = decltype(q_c)::value;
            if constexpr (READ) read_cluster(q_c, Int<1 - S>{}, addr_a, addr_b);
            if constexpr (LOAD) load_cluster(q_c, cur);
            AXONN_FENCE();
            if constexpr (Q < NC - 1)
                mfma_range(s_c, Int<PB + Q * DP>{}, Int<PB + (Q + 1) * DP>{});
            else
                mfma_range(s_c, Int<PB + (NC - 1) * DP>{}, Int<NM>{});
            AXONN_FENCE();
        });
        if constexpr (LOAD) advance_window();
        if constexpr (S == 1) cur ^= BUF;
    };
    using Yes = std::true_type;
    using No = std::false_type;

    // fragments of iteration 0, sub-step 0
    static_for<NC>([&](auto q_c) __attribute__((always_inline)) { read_cluster(q_c, Int<0>{}, raddr_a[0], raddr_b[0]); });
    const int KI = ktotal / Cfg::KS;   // at least 2
    for (int it = KI - 2; it > 0; --it) {
        substep(Int<0>{}, Yes{}, No{});
        substep(Int<1>{}, Yes{}, Yes{});
    }
    substep(Int<0>{}, Yes{}, No{});   // iteration KI-2: nothing left to fetch
    substep(Int<1>{}, Yes{}, No{});
    substep(Int<0>{}, Yes{}, No{});   // iteration KI-1
    substep(Int<1>{}, No{}, No{});
    __syncthreads();   // every wave is done with the buffers before the epilogue reuses LDS

    // ---- split-K exchange: slot element ((wave*MI + i)*NI + j)*64 + lane, 16 bytes each -------------
    if constexpr (SPLITK) {
        const int tiles = tiles_m * tiles_n;
        const size_t in_slot = (size_t)wave * (MI * NI * 64) + lane;
        if (krange != 0) {
            const size_t slot = (size_t)(krange - 1) * tiles + tile_id;
            f32x4* dst = reinterpret_cast<f32x4*>(sk.partials) + slot * (BM * BN / 4) + in_slot;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) dst[(i * NI + j) * 64] = acc[i][j];
            // one device-scope release per workgroup (see gemm_tile_kernel)
            __syncthreads();
            if (t == 0) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                __hip_atomic_store(&sk.flags[slot], sk.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            return;
        }
        for (int r = 1; r < sk.splits; ++r) {
            const size_t slot = (size_t)(r - 1) * tiles + tile_id;
            if (t == 0) {
                uint32_t probes = 0;
                while (__hip_atomic_load(&sk.flags[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != sk.epoch) {
                    if (++probes > kSplitSpinLimit) {
                        atomicAdd(sk.timeouts, 1u);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(32);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }
            __syncthreads();
            const f32x4* src = reinterpret_cast<const f32x4*>(sk.partials) + slot * (BM * BN / 4) + in_slot;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                f32x4 v[NI];
#pragma unroll
                for (int j = 0; j < NI; ++j) v[j] = __builtin_nontemporal_load(src + (i * NI + j) * 64);
                AXONN_FENCE();
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j] += v[j];
                AXONN_FENCE();
            }
        }
    }

    // ---- epilogue: fp32 -> bf16, transpose through this wave's private LDS region --------------
    // acc[i][j][e] = C[m = i*16 + l%16][n = j*16 + 4*(l/16) + e]
    constexpr int CPR = TN / 8;   // 16-byte chunks per row of the wave tile
    constexpr uint32_t CMASK = CPR - 1;
    uint8_t* epi = smem + wave * (TM * TN * 2);
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const uint32_t row = i * 16 + r16;
            const uint32_t chunk = j * 2 + (quad >> 1);
            u32x2 v;
            v[0] = pack2_bf16(acc[i][j][0], acc[i][j][1]);
            v[1] = pack2_bf16(acc[i][j][2], acc[i][j][3]);
            *reinterpret_cast<u32x2*>(epi + row * (TN * 2) + ((chunk ^ (row & CMASK)) << 4) + (quad & 1) * 8) = v;
        }
        AXONN_FENCE();   // convert block row by block row: keeps register pressure low
    }
    __syncthreads();
    uint16_t* pc = C + (m0 + wm * TM) * (int64_t)ldc + n0 + wn * TN;
#pragma unroll
    for (int it = 0; it < (TM * CPR) / 64; ++it) {
        const uint32_t idx = it * 64 + lane;
        const uint32_t row = idx / CPR, ch = idx % CPR;
        const u32x4 v = *reinterpret_cast<const u32x4*>(epi + row * (TN * 2) + ((ch ^ (row & CMASK)) << 4));
        *reinterpret_cast<u32x4*>(pc + (int64_t)row * ldc + ch * 8) = v;
    }
#undef AXONN_FENCE
}

}  // namespace axonn
