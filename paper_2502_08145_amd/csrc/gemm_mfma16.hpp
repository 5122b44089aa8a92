// The tile kernel built on v_mfma_f32_16x16x32_bf16 instead of v_mfma_f32_32x32x16_bf16.
//
// Same data movement as gemm_tile_kernel (LDS ring of 32-k stages filled by direct loads, paired for
// K-contiguous operands; swizzled LDS layouts; split-K; XCD-aware tile order) -- see gemm_mfma.hpp.
// What changes is the matrix instruction and with it the register-level pipeline:
//
//  * On MI355X the 16x16x32 instruction sustains the same peak rate as the 32x32x16 one but draws
//    less power on random data: an MFMA-only loop on N(0,1) operands runs 5-15 % faster with it
//    (higher sustained clock), and this kernel is power-limited.
//  * A fragment is a 16-row block with ALL 32 k of a stage (lane l: row l%16, k = 8*(l/16)..+7), so
//    a K-step is one MFMA "k" and there are no k16 substeps.  The fragments are double-buffered by
//    whole K-steps: while the MFMAs of K-step t run on one register buffer, the fragments of K-step
//    t+1 are read from LDS into the other.  The loop body is two K-steps (buffer 0, buffer 1), so
//    the number of K-steps must be even.
//  * The register buffer is one more pipeline stage: stage t is read during K-step t-1, so it is
//    free for refilling one step earlier, and loads run NS-1 and NS K-steps ahead.
//  * One barrier per K-step, a quarter of the way into the step's MFMAs: every wave has by then
//    the fragments of K-step t in registers (stage t is released) and its share of K-step t+1 has
//    landed (vmcnt), so after it stage t+1 may be read and stage t refilled.
#pragma once
#include "gemm_mfma.hpp"

namespace axonn {

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int BM, int BN, int WM, int WN>
struct TileCfg16 {
    static constexpr int NW = WM * WN;
    static constexpr int NT = 64 * NW;
    static constexpr int TM = BM / WM, TN = BN / WN;        // wave tile
    static constexpr int MI = TM / 16, NI = TN / 16;        // 16x16 blocks per wave tile
    static constexpr int STAGE_BYTES = (BM + BN) * KB * 2;
    // (128 x 128: six stages are 96 KB, one workgroup per compute unit.  Five stages, 80 KB, two per unit,
    // measured 5-17 % faster in NN and TN on outputs of 512 and more small tiles, which the planner gives
    // to the large tile anyway, and 8-10 % slower on the outputs of few tiles and long K that it is
    // picked for.)
    static constexpr int NS = (BM + BN == 512) ? 5 : 6;
    static constexpr int RING_BYTES = NS * STAGE_BYTES;
    static constexpr int EPI_BYTES = BM * BN * 2;
    static constexpr int LDS_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
    static constexpr int NTAIL = NS % 2 ? NS + 1 : NS;      // K-steps outside the main loop (even)
    static constexpr int MIN_K = KB * NTAIL;
    static_assert((BM == 128 || BM == 256) && (BN == 128 || BN == 256), "tile extents are 128 or 256");
    static_assert(WM == 2 && (WN == 2 || WN == 4), "4 or 8 waves");
    static_assert(MI % 4 == 0 && NI % 4 == 0, "fragment waits are tied four blocks at a time");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
};

// Direct loads in flight (see LoadPlan): here every load of a K-step is issued after the step's
// barrier, and at the barrier of step t the loads of the last NS-LAG steps may still be in flight.
// Tail step j is step KT - NTAIL + j; steps before the tail are full.
template <int QA, int QB, bool PAIR_A, bool PAIR_B, int NS, int NTAIL>
struct LoadPlan16 {
    static constexpr int NL = QA + QB;
    static constexpr bool ANY_PAIR = PAIR_A || PAIR_B;
    static constexpr int LAG = ANY_PAIR ? 3 : 2;
    static constexpr int issued(int kind) {
        return kind == 2 ? NL : kind == 1 ? (PAIR_A ? QA / 2 : 0) + (PAIR_B ? QB / 2 : 0) : 0;
    }
    // step t fetches K-steps t+NS-1 (paired operands) and t+NS: full while t+NS <= KT-1
    static constexpr int tail_kind(int j) {
        const int from_end = NTAIL - j;            // t = KT - from_end
        return from_end > NS ? 2 : (from_end == NS && ANY_PAIR) ? 1 : 0;
    }
    static constexpr int tail_vm(int j) {
        int n = 0;
        for (int s = j - (NS - LAG); s < j; ++s) n += issued(s < 0 ? 2 : tail_kind(s));
        return n;
    }
    static constexpr int PROLOGUE_VM = (NS - (ANY_PAIR ? 2 : 1)) * NL;   // K-step 0 has landed
};

// ---- shared by the kernels whose accumulators are 16x16 blocks: acc[i][j][e] = C[m = i*16 + l%16]
// [n = j*16 + 4*(l/16) + e] of the wave tile ------------------------------------------------------------

// Split-K exchange (see SplitK).  Slot element ((wave*MI + i)*NI + j)*64 + lane, 16 bytes each.  Returns
// true for the workgroups of K ranges 1.. (they are done); the range-0 workgroup returns false with
// the other ranges added to its accumulators, in range order.
template <int BM, int BN, int MI, int NI>
__device__ __forceinline__ bool split_k_exchange16(f32x4 (&acc)[MI][NI], const SplitK& sk, int krange, int tile_id,
                                                   int tiles, int wave, int lane, int t) {
    // the lane number through an opaque move: what is derived from it here is then computed here, after
    // the K loop, instead of being hoisted above it and kept (or spilled) across it
    asm volatile("" : "+v"(lane));
    const size_t in_slot = (size_t)wave * (MI * NI * 64) + lane;
    if (krange != 0) {
        const size_t slot = (size_t)(krange - 1) * tiles + tile_id;
        f32x4* dst = reinterpret_cast<f32x4*>(sk.partials) + slot * (BM * BN / 4) + in_slot;
        // device-scope stores: they go through the L2 to memory as they are issued, instead of sitting in
        // the L2 until the release below writes the whole cache back (release 3.8 -> 0.8 us, the reader's
        // wait for the flag 9.3 -> 6.5 us).  The s_nop is the wait state this chip wants between a store
        // of more than 8 bytes and a VALU write to its data registers: the compiler inserts it behind its
        // own stores, but cannot see this one (where the accumulators live in AGPRs the next instruction
        // is the copy of the next block into the same registers).
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 0" ::"v"(dst + (i * NI + j) * 64), "v"(acc[i][j]) : "memory");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // acknowledged: the compiler does not count stores issued from asm
        // Cache maintenance is dear on a chip of eight private L2s (a device-scope release writes the
        // L2 back, an acquire invalidates it), so each workgroup does it once: the barrier orders
        // every thread's stores before thread 0's release, and thread 0's acquire before every
        // thread's loads.
        __syncthreads();
        if (t == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __hip_atomic_store(&sk.flags[slot], sk.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return true;
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
                __builtin_amdgcn_s_sleep(4);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // no stale cached copy of the slot
            // The slot is as good as consumed (its writer does not touch the flag again): take the flag down.
            // A launch replayed from a captured HIP graph carries the epoch of its capture, and must not
            // find that value left over from the replay before.
            __hip_atomic_store(&sk.flags[slot], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const f32x4* src = reinterpret_cast<const f32x4*>(sk.partials) + slot * (BM * BN / 4) + in_slot;
        // The slot comes from memory (the writer's L2 has written it back), a trip of a microsecond or
        // two, so as many loads as there are registers for are in flight together: RB rows of blocks at a
        // time, 64 registers, which the fragments no longer need (one row at a time, eight trips for a
        // large tile instead of two, made the exchange of two K ranges 8 us longer).
        constexpr int RB = MI % 4 == 0 ? 4 : MI % 2 == 0 ? 2 : 1;
#pragma unroll
        for (int i0 = 0; i0 < MI; i0 += RB) {
            f32x4 v[RB][NI];
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) v[i][j] = __builtin_nontemporal_load(src + ((i0 + i) * NI + j) * 64);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i0 + i][j] += v[i][j];
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    return false;
}

// Epilogue: fp32 -> bf16 (round to nearest even, once), transposed through this wave's private LDS
// region (TM x TN bf16 at smem + wave * TM*TN*2; all waves must be done with the operand buffers),
// 16-byte coalesced non-temporal stores (see flush_c_block for why non-temporal).  `pc` points at the
// wave tile's first element in C.  Streaming the tile out block row by block row, instead of staging
// all of it, waiting at a workgroup barrier and then storing, took 2 % off the 8-wave TN kernel at
// K = 2048 (the stores start eight times earlier).
template <int TM, int TN, int MI, int NI>
__device__ __forceinline__ void store_tile16(f32x4 (&acc)[MI][NI], uint8_t* smem, uint16_t* pc, int ldc, int wave, int lane) {
    asm volatile("" : "+v"(lane));   // see split_k_exchange16: keeps the epilogue's addresses out of the K loop's registers
    constexpr int CPR = TN / 8;   // 16-byte chunks per row of the wave tile (8 or 16)
    constexpr uint32_t CMASK = CPR - 1;
    const uint32_t quad = lane >> 4, r16 = lane & 15;
    uint8_t* epi = smem + wave * (TM * TN * 2);
    // a block row (16 rows of the wave tile) at a time: staged, read back by rows and stored while the
    // next one is converted.  The region is this wave's own and a wave's LDS operations execute in
    // order, so no barrier is needed between the staging writes and the reads.
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
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int it = 0; it < (16 * CPR) / 64; ++it) {
            const uint32_t idx = it * 64 + lane;
            const uint32_t row = i * 16 + idx / CPR, ch = idx % CPR;
            const u32x4 v = *reinterpret_cast<const u32x4*>(epi + row * (TN * 2) + ((ch ^ (row & CMASK)) << 4));
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(pc + (int64_t)row * ldc + ch * 8));
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// One block row of a wave tile (16 rows x TN columns, acc[i][0..NI)) to C at `pc_row`, converted and
// transposed like store_tile16 does it, through a region of 16 * TN * 2 bytes at `epi` that belongs to
// this wave alone.  The region may be reused for the next block row straight away: a wave's LDS
// operations execute in order, so the next staging writes cannot overtake these reads.
template <int TN, int NI>
__device__ __forceinline__ void store_block_row16(f32x4 (&row)[NI], uint8_t* epi, uint16_t* pc_row, int ldc, int lane) {
    constexpr int CPR = TN / 8;
    constexpr uint32_t CMASK = CPR - 1;
    const uint32_t quad = lane >> 4, r16 = lane & 15;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const uint32_t chunk = j * 2 + (quad >> 1);
        u32x2 v;
        v[0] = pack2_bf16(row[j][0], row[j][1]);
        v[1] = pack2_bf16(row[j][2], row[j][3]);
        *reinterpret_cast<u32x2*>(epi + r16 * (TN * 2) + ((chunk ^ (r16 & CMASK)) << 4) + (quad & 1) * 8) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int it = 0; it < (16 * CPR) / 64; ++it) {
        const uint32_t idx = it * 64 + lane;
        const uint32_t r = idx / CPR, ch = idx % CPR;
        const u32x4 v = *reinterpret_cast<const u32x4*>(epi + r * (TN * 2) + ((ch ^ (r & CMASK)) << 4));
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(pc_row + (int64_t)r * ldc + ch * 8));
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Requires M % BM == 0, N % BN == 0, K % 64 == 0, K >= TileCfg16::MIN_K (per K range when split).
template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, bool SPLITK>
__global__ __launch_bounds__(64 * WM * WN) void gemm_tile_kernel16(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
    int K, int lda, int ldb, int ldc, int tiles_m, int tiles_n, int group_m, SplitK sk) {
    using Cfg = TileCfg16<BM, BN, WM, WN>;
    constexpr int NW = Cfg::NW;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, MI = Cfg::MI, NI = Cfg::NI, NS = Cfg::NS, NTAIL = Cfg::NTAIL;
    constexpr uint32_t SB = Cfg::STAGE_BYTES, RING = Cfg::RING_BYTES;
    // The full-rate layout of the transposing reads (TR16) pays in the 8-wave kernel when it is B alone
    // that is read that way (NN: +2-3 %); with both operands MN-contiguous (TN) it measured 2 % slower
    // than the old one, and so did the 4-wave NN kernels (1-2 %).
    using OpA = typename std::conditional<A_KC, OperandKContig<BM, 0, NW, MI / 2, 1>, OperandMNContig<BM, 0, NW, MI / 2>>::type;
    using OpB = typename std::conditional<B_KC, OperandKContig<BN, BM * KB * 2, NW, NI / 2, 1>,
                                          OperandMNContig<BN, BM * KB * 2, NW, NI / 2, (A_KC && NW == 8)>>::type;
    constexpr int QA = OpA::QL, QB = OpB::QL;                  // direct loads per wave per stage
    constexpr int NM = MI * NI;                                // MFMAs per K-step
    static_assert(NM % 8 == 0, "the step is cut in quarters and eighths");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- workgroup -> output tile and K range ------------------------------------------------
    const TileWork work = map_workgroup<SPLITK, BM * BN == 256 * 256>(blockIdx.x, gridDim.x, K, tiles_m, tiles_n, group_m, sk);
    const int tile_m = work.tile_m, tile_n = work.tile_n, krange = work.krange, ktotal = work.ktotal;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

    const uint32_t lds0 = lds_address(smem);
    OpA opa;
    OpB opb;
    const int64_t k0 = (int64_t)krange * ktotal;
    // the load schedule starts NS K-steps before K-step 0
    constexpr bool FIRST_ODD = NS % 2 == 1;
    opa.init(A + (A_KC ? k0 : k0 * lda), m0, 2u * (uint32_t)lda, lane, wave, lds0, wm * TM, FIRST_ODD);
    opb.init(B + (B_KC ? k0 : k0 * ldb), n0, 2u * (uint32_t)ldb, lane, wave, lds0, wn * TN, FIRST_ODD);

    f32x4 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // fragment double buffer: [K-step parity][16-row block]; pinned registers (see lds_read128)
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
    auto mfma = [&](auto buf_c, auto idx_c) __attribute__((always_inline)) {
        // block rows in order, the blocks of a row back and forth: from one MFMA to the next exactly one
        // operand changes (less toggling on the operand buses of a power-limited chip)
        constexpr int BUF = decltype(buf_c)::value, I = decltype(idx_c)::value / NI, J0 = decltype(idx_c)::value % NI;
        constexpr int J = (I & 1) ? NI - 1 - J0 : J0;
        acc[I][J] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[BUF][J].get(), fa[BUF][I].get(), acc[I][J], 0, 0, 0);
    };
    auto mfma_range = [&](auto buf_c, auto lo_c, auto hi_c) __attribute__((always_inline)) {
        constexpr int LO = decltype(lo_c)::value, HI = decltype(hi_c)::value;
        static_for<HI - LO>([&](auto d) __attribute__((always_inline)) { mfma(buf_c, Int<LO + decltype(d)::value>{}); });
    };
    // All LDS reads issued so far have landed (fragment registers tied to the wait, four at a time).
    auto wait_fragments = [&](auto buf_c) __attribute__((always_inline)) {
        constexpr int BUF = decltype(buf_c)::value;
        static_for<MI / 4>([&](auto d) __attribute__((always_inline)) { tie_to_lds_wait<4>(&fa[BUF][4 * decltype(d)::value]); });
        static_for<NI / 4>([&](auto d) __attribute__((always_inline)) { tie_to_lds_wait<4>(&fb[BUF][4 * decltype(d)::value]); });
    };
    // Quarter Q (0..3) of the fragment reads of a stage into buffer BUF: the MI + NI blocks (A first)
    // are dealt out evenly.
    auto read_cluster = [&](auto q_c, auto buf_c, const typename OpA::Cursor16& ca, const typename OpB::Cursor16& cb) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value, BUF = decltype(buf_c)::value;
        constexpr int NBLK = MI + NI, FIRST = Q * NBLK / 4, LAST = (Q + 1) * NBLK / 4;
        static_for<LAST - FIRST>([&](auto d) __attribute__((always_inline)) {
            constexpr int X = FIRST + decltype(d)::value;
            if constexpr (X < MI)
                opa.template read16<X>(fa[BUF][X], ca);
            else
                opb.template read16<X - MI>(fb[BUF][X - MI], cb);
        });
    };
    // Direct loads (see gemm_tile_kernel): during K-step t, after its barrier, a plain operand fetches
    // K-step t+NS into the stage just released ("far"), a paired operand half its row groups for
    // K-steps t+NS-1 and t+NS into the stages "near" (released one step earlier) and "far".
    auto issue_loads = [&](auto op_c, auto kind_c, auto half_c, uint32_t st_near, uint32_t st_far) __attribute__((always_inline)) {
        constexpr bool IS_A = decltype(op_c)::value == 0;
        constexpr int KIND = decltype(kind_c)::value, H = decltype(half_c)::value;
        using Op = typename std::conditional<IS_A, OpA, OpB>::type;
        auto& op = [&]() __attribute__((always_inline)) -> auto& { if constexpr (IS_A) return opa; else return opb; }();
        constexpr int NB = Op::NBASE, FIRST = H == 0 ? 0 : (NB + 1) / 2, LAST = H == 0 ? (NB + 1) / 2 : NB;
        static_for<LAST - FIRST>([&](auto d) __attribute__((always_inline)) {
            constexpr int X = FIRST + decltype(d)::value;
            if constexpr (Op::PAIR) {
                if constexpr (KIND >= 1) op.template issue<X, 0>(st_near);
                if constexpr (KIND == 2) op.template issue<X, 1>(st_far);
            } else {
                if constexpr (KIND == 2) op.template issue<X, 0>(st_far);
            }
        });
    };
    using Plan = LoadPlan16<QA, QB, OpA::PAIR, OpB::PAIR, NS, NTAIL>;
    auto next_stage = [&](uint32_t off) __attribute__((always_inline)) -> uint32_t { return off + SB == RING ? 0u : off + SB; };

    // ---- prologue: the loads "steps -NS .. -1" would have issued: K-steps 0 .. NS-1 ---------------
    static_for<NS>([&](auto v) __attribute__((always_inline)) {
        constexpr int T = decltype(v)::value - NS;                // virtual step
        constexpr uint32_t FAR = (T + NS) * SB;                   // stage of K-step T+NS
        static_for<2>([&](auto op_c) __attribute__((always_inline)) {
            constexpr bool IS_A = decltype(op_c)::value == 0;
            using Op = typename std::conditional<IS_A, OpA, OpB>::type;
            auto& op = [&]() __attribute__((always_inline)) -> auto& { if constexpr (IS_A) return opa; else return opb; }();
            if constexpr (Op::PAIR && T == -NS) {
                // K-step -1 does not exist: only the K-step 0 half of the pair, window stays
                static_for<Op::NBASE>([&](auto d) __attribute__((always_inline)) { op.template issue<decltype(d)::value, 0>(FAR); });
                op.flip();
            } else {
                constexpr uint32_t NEAR = Op::PAIR ? FAR - SB : 0u;
                issue_loads(op_c, Int<2>{}, Int<0>{}, NEAR, FAR);
                issue_loads(op_c, Int<2>{}, Int<1>{}, NEAR, FAR);
                op.advance();
            }
        });
    });
    wait_vmcnt<Plan::PROLOGUE_VM>();
    __builtin_amdgcn_s_barrier();
    AXONN_FENCE();
    // stage of the K-step whose fragments are read next, and the two stages being refilled
    uint32_t st_read = 0, st_near = (NS - 1) * SB, st_far = 0;
    typename OpA::Cursor16 ca = opa.cursor16(st_read);
    typename OpB::Cursor16 cb = opb.cursor16(st_read);

    // ---- one K-step: MFMAs on buffer BUF, fragments of the next K-step into the other buffer -------
    //   KIND: what it fetches (2 all, 1 only the K-step t+NS-1 halves of paired operands, 0 nothing).
    //   NEXT: a following K-step exists.   VM: loads that may still be in flight at the barrier.
    //   PHASE: waves 4..7 of an 8-wave workgroup issue their clusters an eighth of a step later.
    auto step = [&](auto phase_c, auto buf_c, auto kind_c, auto next_c, auto vm_c) __attribute__((always_inline)) {
        constexpr bool NEXT = decltype(next_c)::value;
        constexpr int VM = decltype(vm_c)::value, KIND = decltype(kind_c)::value, BUF = decltype(buf_c)::value;
        constexpr int PB = NM / 8;                                       // MFMAs before the barrier
        constexpr int P0 = PB + (decltype(phase_c)::value ? NM / 8 : 0);   // ... before cluster 0
        constexpr int DP = (3 * NM / 4 - P0) / 3;                        // between clusters; the last quarter of
                                                                         // the step covers the latency of the last reads
        wait_fragments(buf_c);
        AXONN_FENCE();
        mfma_range(buf_c, Int<0>{}, Int<PB>{});
        AXONN_FENCE();
        if constexpr (NEXT) {
            wait_vmcnt<VM>();
            __builtin_amdgcn_s_barrier();
            AXONN_FENCE();
            ca = opa.cursor16(st_read);
            cb = opb.cursor16(st_read);
        }
        mfma_range(buf_c, Int<PB>{}, Int<P0>{});
        AXONN_FENCE();
        if constexpr (NEXT) read_cluster(Int<0>{}, Int<1 - BUF>{}, ca, cb);
        issue_loads(Int<0>{}, kind_c, Int<0>{}, st_near, st_far);
        AXONN_FENCE();
        mfma_range(buf_c, Int<P0>{}, Int<P0 + DP>{});
        AXONN_FENCE();
        if constexpr (NEXT) read_cluster(Int<1>{}, Int<1 - BUF>{}, ca, cb);
        issue_loads(Int<0>{}, kind_c, Int<1>{}, st_near, st_far);
        AXONN_FENCE();
        mfma_range(buf_c, Int<P0 + DP>{}, Int<P0 + 2 * DP>{});
        AXONN_FENCE();
        if constexpr (NEXT) read_cluster(Int<2>{}, Int<1 - BUF>{}, ca, cb);
        issue_loads(Int<1>{}, kind_c, Int<0>{}, st_near, st_far);
        AXONN_FENCE();
        mfma_range(buf_c, Int<P0 + 2 * DP>{}, Int<P0 + 3 * DP>{});
        AXONN_FENCE();
        if constexpr (NEXT) read_cluster(Int<3>{}, Int<1 - BUF>{}, ca, cb);
        issue_loads(Int<1>{}, kind_c, Int<1>{}, st_near, st_far);
        if constexpr (KIND == 2) {
            opa.advance();
            opb.advance();
        }
        AXONN_FENCE();
        mfma_range(buf_c, Int<P0 + 3 * DP>{}, Int<NM>{});
        AXONN_FENCE();
        st_near = st_far;
        st_far = next_stage(st_far);
        st_read = next_stage(st_read);
    };
    using Yes = std::true_type;

    const int KT = ktotal / KB;   // even, at least NTAIL
    auto main_loop = [&](auto phase_c) __attribute__((always_inline)) {
        // fragments of K-step 0 (inside the phase's own code path: no join between a read and its wait)
        read_cluster(Int<0>{}, Int<0>{}, ca, cb);
        read_cluster(Int<1>{}, Int<0>{}, ca, cb);
        read_cluster(Int<2>{}, Int<0>{}, ca, cb);
        read_cluster(Int<3>{}, Int<0>{}, ca, cb);
        st_read = SB;   // K-step 1 is read during step 0
        constexpr int VM_FULL = Plan::tail_vm(-1);
        for (int kt = (KT - NTAIL) / 2; kt > 0; --kt) {
            step(phase_c, Int<0>{}, Int<2>{}, Yes{}, Int<VM_FULL>{});
            step(phase_c, Int<1>{}, Int<2>{}, Yes{}, Int<VM_FULL>{});
        }
        static_for<NTAIL>([&](auto j_c) __attribute__((always_inline)) {
            constexpr int J = decltype(j_c)::value;
            step(phase_c, Int<J % 2>{}, Int<Plan::tail_kind(J)>{}, std::integral_constant<bool, (J + 1 < NTAIL)>{},
                 Int<Plan::tail_vm(J)>{});
        });
    };
    if constexpr (NW == 8) {
        if (wave >= 4) main_loop(Int<1>{});   // wave-uniform; both paths hit the same barriers
        else main_loop(Int<0>{});
    } else {
        main_loop(Int<0>{});
    }
    __syncthreads();   // every wave is done with the ring before the epilogue reuses LDS

    if constexpr (SPLITK) {
        if (split_k_exchange16<BM, BN, MI, NI>(acc, sk, krange, work.tile_id, tiles_m * tiles_n, wave, lane, t)) return;
    }
    store_tile16<TM, TN, MI, NI>(acc, smem, C + (m0 + wm * TM) * (int64_t)ldc + n0 + wn * TN, ldc, wave, lane);
#undef AXONN_FENCE
}

}  // namespace axonn
