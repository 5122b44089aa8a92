// The tile kernel with LDS stages of 64 k and one barrier per 64 k, four or eight waves, tiles of 256 x 256,
// 256 x 128 and 128 x 256.
//
// Why a kernel of its own.  In gemm_tile_kernel16 a K-contiguous operand is staged 32 k at a time:
// a row of a stage is 64 bytes, half a cache line, so every direct load asks the L1 for sixteen
// half lines, and there is a barrier every 32 k.  Here:
//
//  * a K-contiguous panel is staged 64 k at a time: an LDS row is one whole 128-byte line (row r,
//    the eight 16-byte chunks XOR-swizzled by (r>>1)&7: ds_read_b128 of sixteen consecutive rows
//    then touches every bank once), a direct load fetches 8 rows x 128 B: eight full-line requests
//    instead of sixteen half-line ones.  An MN-contiguous panel is two 32-k stages of
//    OperandMNContig side by side;
//  * per operand two buffers of BM (BN) x 64 k (256 x 256: 2 x 64 KB in all); 2 x 2 waves (every LDS
//    byte is read twice, not three times) or 2 x 4 waves (256 x 256: wave tile 128 x 64, two waves per SIMD);
//  * ONE barrier per 64 k.  An iteration is two sub-steps of 32 k.  During sub-step 0 of iteration i
//    the fragments of its sub-step 1 are read; during sub-step 1, after the barrier, the fragments
//    of iteration i+1 (other buffer), and the direct loads of iteration i+2 go out into the buffer
//    that iteration i has just finished with.  At the barrier every load issued so far must have
//    landed (vmcnt(0)): those of iteration i+1, issued one iteration earlier, i.e. a lead of
//    almost two sub-steps;
//  * optionally (SCHED 1 or 2) one operand gets a THIRD buffer (160 KB in all) and its loads move to
//    sub-step 0: the buffer they go to was released at the previous iteration's barrier, they have
//    three sub-steps to land, and the load path (which delivers some 52 bytes a clock per compute
//    unit, so the 64 KB of an iteration keep it busy for most of one sub-step) carries half an
//    iteration's bytes in either sub-step instead of all of them in one.  At the barrier the loads
//    that sub-step 0 has just issued may still be in flight (vmcnt(QL): loads complete in order).
//    Which modes gain from it is a measurement (see kernels_k64.hip).
//
// Measured: with eight waves it is the fastest kernel in all three modes (NN and NT: 3-4 % over the
// 32-k kernel in the benchmark step, more for the split-K forms; TN: 2-4 % since C is streamed out as
// non-temporal stores, with the reads and loads of a sub-step cut into six clusters instead of four);
// the 32-k ring keeps TN with four and more K ranges.  On the 256 x 256 tile four waves win only for NT
// without split-K, by a hair (not instantiated); the half tiles run with four.  Fragments, MFMA order (mfma(Bfrag, Afrag)), accumulator
// layout, split-K exchange, epilogue and the XCD-aware tile order are those of gemm_tile_kernel16.
// (TN without split-K takes the epilogue into its last sub-step, see OVERLAP_EPI below.)
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

// Operand policies of the 64-k kernel: a wave issues eight direct loads per operand and iteration.
//   issue<X>(buf)        load X (0..7) of the iteration at the global window, into the buffer at buf
//   advance()            window one iteration (64 k) on
//   cursor(S, buf)       read addresses for sub-step S of that buffer
//   read<I>(frag, cur)   fragment of 16-row block I
template <int ROWS, int REGION, int NW>
struct OperandK64KContig {   // global P[row * ld + k]; LDS [row][64 k], chunks swizzled by (row>>1)&7
    static constexpr int QL = ROWS / 8 / NW;   // loads per wave and iteration: row groups QL*wave .. (8 rows each)
    using Frag = Frag128;
    struct Cursor {
        uint32_t a;
    };
    const uint8_t* base[QL];  // uniform: row group QL*wave + c, k = 0
    uint32_t lds_dst;         // uniform: destination of group QL*wave inside buffer 0
    uint32_t voff[2];         // per lane, [group parity]: row-in-group * ld + fetched chunk * 16 + window
    uint32_t raddr[2];        // [sub-step]: read address of block 0 in buffer 0

    // Lane l of a load lands at (row l/8, slot l%8) of its group; slot s of row r holds chunk
    // s ^ ((r>>1)&7), and (r>>1)&7 = 4*(group&1) + l/16.  A reader lane wants, for block I and
    // sub-step S, row 16*I + l%16 and chunk 4*S + l/16, found in slot (4*S + l/16) ^ ((l%16)>>1);
    // block I is an immediate offset of I * 2048.
    __device__ __forceinline__ void init(const uint16_t* P, int64_t row0, uint32_t ld_bytes, int lane, int wave,
                                         uint32_t lds0, int wave_row_base) {
        static_assert(QL % 2 == 0, "a wave's first row group is an even one");
#pragma unroll
        for (int c = 0; c < QL; ++c)
            base[c] = reinterpret_cast<const uint8_t*>(P) + (size_t)(row0 + 8 * (QL * wave + c)) * ld_bytes;
        lds_dst = lds0 + REGION + (uint32_t)(QL * wave) * 1024u;
        const uint32_t r16 = lane & 15, quad = lane >> 4;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            voff[p] = (uint32_t)(lane >> 3) * ld_bytes + ((((uint32_t)lane & 7u) ^ (4u * p + quad)) << 4);
            raddr[p] = lds0 + REGION + (uint32_t)(wave_row_base + r16) * 128u + (((4u * p + quad) ^ (r16 >> 1)) << 4);
        }
    }
    template <int X>
    __device__ __forceinline__ void issue(uint32_t buf) const {
        direct_load16(lds_dst + buf + X * 1024u, base[X], voff[X & 1]);
    }
    __device__ __forceinline__ void advance() {
        voff[0] += 128;
        voff[1] += 128;
    }
    // The window back to k = 0 (it has advanced `k_bytes`) of the panel rows that start at row0.
    __device__ __forceinline__ void retarget(const uint16_t* P, int64_t row0, uint32_t ld_bytes, int wave, uint32_t k_bytes) {
#pragma unroll
        for (int c = 0; c < QL; ++c)
            base[c] = reinterpret_cast<const uint8_t*>(P) + (size_t)(row0 + 8 * (QL * wave + c)) * ld_bytes;
        voff[0] -= k_bytes;
        voff[1] -= k_bytes;
    }
    template <int S>
    __device__ __forceinline__ Cursor cursor(uint32_t buf) const {
        return Cursor{raddr[S] + buf};
    }
    template <int I>
    __device__ __forceinline__ void read(Frag& f, const Cursor& c) const {
        lds_read128<I * 2048>(f.v, c.a);
    }
};

template <int ROWS, int REGION, int NW, int NB>
struct OperandK64MNContig {   // global P[k * ld + row]; the buffer holds two 32-k stages of OperandMNContig
    using Inner = OperandMNContig<ROWS, REGION, NW, NB>;
    static constexpr int QH = Inner::QL;   // loads per wave and 32-k stage
    static constexpr int QL = 2 * QH;
    using Frag = typename Inner::Frag;
    using Cursor = typename Inner::Cursor16;
    static constexpr uint32_t HALF = ROWS * KB * 2;   // bytes of one 32-k stage
    Inner in;
    uint32_t voff_hi[QH];     // the loads of the second stage: 32 k-rows on

    __device__ __forceinline__ void init(const uint16_t* P, int64_t row0, uint32_t ld_bytes, int lane, int wave,
                                         uint32_t lds0, int wave_row_base) {
        in.init(P, row0, ld_bytes, lane, wave, lds0, wave_row_base, false);
#pragma unroll
        for (int c = 0; c < QH; ++c) voff_hi[c] = in.voff[c] + (uint32_t)in.kstep_bytes;   // fits: ld < 2^24
    }
    template <int X>
    __device__ __forceinline__ void issue(uint32_t buf) const {
        constexpr int C = X % QH;
        if constexpr (X < QH)
            direct_load16(in.lds_dst[C] + buf, in.base, in.voff[C]);
        else
            direct_load16(in.lds_dst[C] + buf + HALF, in.base, voff_hi[C]);
    }
    __device__ __forceinline__ void advance() {
        in.base += 2 * in.kstep_bytes;   // 64-bit: panels may exceed 4 GB
    }
    // The window back to k = 0 of the panel rows (m or n) that start at row0.
    __device__ __forceinline__ void retarget(const uint16_t* P, int64_t row0, uint32_t ld_bytes, int wave, uint32_t /*k_bytes*/) {
        in.base = reinterpret_cast<const uint8_t*>(P) + (size_t)row0 * 2 + (size_t)(Inner::KR * Inner::QL * wave) * ld_bytes;
    }
    template <int S>
    __device__ __forceinline__ Cursor cursor(uint32_t buf) const {
        return in.cursor16(buf + S * HALF);
    }
    template <int I>
    __device__ __forceinline__ void read(Frag& f, const Cursor& c) const {
        in.template read16<I>(f, c);
    }
};

// Load schedules of gemm_tile_kernel_k64 (SCHED):
//   0  two buffers per operand; all loads of an iteration in sub-step 1, into the running buffers
//   1  three A buffers, A's loads in sub-step 0; B as in 0
//   2  three B buffers, B's loads in sub-step 0; A as in 0
//   3  three buffers each (fits for the 128 x 256 and 256 x 128 tiles); half of an iteration's loads in
//      either sub-step
constexpr int k64_a_buffers(int sched) { return (sched == 1 || sched == 3) ? 3 : 2; }
constexpr int k64_b_buffers(int sched) { return (sched == 2 || sched == 3) ? 3 : 2; }
constexpr int k64_lds_bytes(int bm, int bn, int sched) {
    const int ring = (k64_a_buffers(sched) * bm + k64_b_buffers(sched) * bn) * TileCfgK64::KS * 2, epi = bm * bn * 2;
    return ring > epi ? ring : epi;
}

// Requires M % BM == 0, N % BN == 0, K % 64 == 0, K >= 128 (per K range when split).
template <int BM, int BN, int WN, bool A_KC, bool B_KC, bool SPLITK, int SCHED>
__global__ __launch_bounds__(128 * WN) void gemm_tile_kernel_k64(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
    int K, int lda, int ldb, int ldc, int tiles_m, int tiles_n, int group_m, SplitK sk) {
    using Cfg = TileCfgK64;
    static_assert(WN == 2 || WN == 4, "2 x 2 or 2 x 4 waves");
    static_assert((BM == 128 || BM == 256) && (BN == 128 || BN == 256), "tile extents are 128 or 256");
    constexpr int NW = 2 * WN;
    constexpr int TM = BM / 2, TN = BN / WN, MI = TM / 16, NI = TN / 16, NM = MI * NI;
    static_assert(SCHED >= 0 && SCHED <= 3, "load schedule");
    constexpr int NAB = k64_a_buffers(SCHED), NBB = k64_b_buffers(SCHED);
    constexpr uint32_t ABUF = BM * Cfg::KS * 2, BBUF = BN * Cfg::KS * 2, REGION_B = NAB * ABUF;
    static_assert(k64_lds_bytes(BM, BN, SCHED) <= 160 * 1024, "LDS per workgroup");
    constexpr int NRD = MI + NI;   // fragment reads per wave and sub-step
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- workgroup -> output tile and K range ------------------------------------------------
    const TileWork work = map_workgroup<SPLITK, BM * BN == 256 * 256>(blockIdx.x, gridDim.x, K, tiles_m, tiles_n, group_m, sk);
    const int tile_m = work.tile_m, tile_n = work.tile_n, krange = work.krange;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    int ktotal = work.ktotal;
    int64_t k0 = (int64_t)krange * ktotal;
    if constexpr (SPLITK) {
        // the writers' ranges are a little shorter than the reader's: their partial tiles are on their
        // way while the reader still multiplies
        if (krange == 0) {
            ktotal += (sk.splits - 1) * sk.skew;
        } else {
            ktotal -= sk.skew;
            k0 = (int64_t)work.ktotal + (int64_t)(sk.splits - 1) * sk.skew + (int64_t)(krange - 1) * ktotal;
        }
    }

    // ---- operands ------------------------------------------------------------------------------------
    using OpA = typename std::conditional<A_KC, OperandK64KContig<BM, 0, NW>, OperandK64MNContig<BM, 0, NW, MI / 2>>::type;
    using OpB = typename std::conditional<B_KC, OperandK64KContig<BN, REGION_B, NW>, OperandK64MNContig<BN, REGION_B, NW, NI / 2>>::type;
    constexpr int QLA = OpA::QL, QLB = OpB::QL, NLD = QLA + QLB;   // direct loads per wave and iteration
    static_assert(QLA == BM / 2 / NW / 4 && QLB == BN / 2 / NW / 4, "a load is 1 KB of a panel of BM (BN) x 64 bf16");
    const uint32_t lds0 = lds_address(smem);
    OpA opa;
    OpB opb;
    opa.init(A + (A_KC ? k0 : k0 * lda), m0, 2u * (uint32_t)lda, lane, wave, lds0, wm * TM);
    opb.init(B + (B_KC ? k0 : k0 * ldb), n0, 2u * (uint32_t)ldb, lane, wave, lds0, wn * TN);
    // load number X (0 .. QL-1) of an operand's panel of one iteration into the buffer at `buf`
    auto issue_a = [&](auto x_c, uint32_t buf) __attribute__((always_inline)) { opa.template issue<decltype(x_c)::value>(buf); };
    auto issue_b = [&](auto x_c, uint32_t buf) __attribute__((always_inline)) { opb.template issue<decltype(x_c)::value>(buf); };

    f32x4 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    typename OpA::Frag fa[2][MI];   // [sub-step][block]; pinned registers (see lds_read128)
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
    // cluster Q of NC: its share of the fragment reads of a sub-step into register buffer S (A
    // blocks, then B), and of the direct loads of an iteration
    // (measured: with two MN-contiguous operands, whose fragments take two transposing reads each, six
    // clusters are 1.5-2 % faster than four; with K-contiguous operands it makes no difference)
    constexpr int NC = (!A_KC && !B_KC) ? 6 : 4;
    constexpr int PB = NM / 8;                          // MFMAs before the barrier and the first cluster
    auto read_cluster = [&](auto q_c, auto s_c, const typename OpA::Cursor& ca, const typename OpB::Cursor& cb) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value, S = decltype(s_c)::value;
        constexpr int RF = Q * NRD / NC, RL = (Q + 1) * NRD / NC;
        static_for<RL - RF>([&](auto d) __attribute__((always_inline)) {
            constexpr int X = RF + decltype(d)::value;
            if constexpr (X < MI)
                opa.template read<X>(fa[S][X], ca);
            else
                opb.template read<X - MI>(fb[S][X - MI], cb);
        });
    };
    // cluster Q's share of the loads that go out in sub-step S.  The loads of an iteration are numbered
    // A's first (0 .. QLA-1), then B's; sub-step S issues LS of them from number LO on.
    auto load_cluster = [&](auto q_c, auto s_c, uint32_t abuf, uint32_t bbuf) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value, S = decltype(s_c)::value;
        constexpr int LO = SCHED == 0 ? 0 : SCHED == 1 ? (S == 0 ? 0 : QLA) : SCHED == 2 ? (S == 0 ? QLA : 0) : (S == 0 ? 0 : NLD / 2);
        constexpr int LS = SCHED == 0 ? (S == 0 ? 0 : NLD)
                         : SCHED == 1 ? (S == 0 ? QLA : QLB)
                         : SCHED == 2 ? (S == 0 ? QLB : QLA)
                                      : (S == 0 ? NLD / 2 : NLD - NLD / 2);
        constexpr int LF = LO + Q * LS / NC, LL = LO + (Q + 1) * LS / NC;
        static_for<LL - LF>([&](auto d) __attribute__((always_inline)) {
            constexpr int X = LF + decltype(d)::value;
            if constexpr (X < QLA)
                issue_a(Int<X>{}, abuf);
            else
                issue_b(Int<X - QLA>{}, bbuf);
        });
    };

    // ---- prologue: iterations 0 and 1 into the first two buffers of each operand ---------------------
    static_for<QLA>([&](auto x) __attribute__((always_inline)) { issue_a(x, 0u); });
    static_for<QLB>([&](auto x) __attribute__((always_inline)) { issue_b(x, 0u); });
    opa.advance();
    opb.advance();
    static_for<QLA>([&](auto x) __attribute__((always_inline)) { issue_a(x, ABUF); });
    static_for<QLB>([&](auto x) __attribute__((always_inline)) { issue_b(x, BBUF); });
    opa.advance();
    opb.advance();
    wait_vmcnt<NLD>();   // iteration 0 has landed
    __builtin_amdgcn_s_barrier();
    AXONN_FENCE();

    // byte offsets of the A buffers of the running iteration, the next one and the one after, and of
    // the running iteration's B buffer (the other one is the next iteration's)
    uint32_t a0 = 0, a1 = ABUF, a2 = NAB == 3 ? 2 * ABUF : 0, b0 = 0, b1 = BBUF, b2 = NBB == 3 ? 2 * BBUF : 0;
    // One sub-step S of the running iteration.
    //   READ: fragments for the following sub-step are read (S = 0: sub-step 1 of the same buffers;
    //         S = 1: sub-step 0 of the next iteration's buffers, after the barrier).
    //   LOAD: the panels of the iteration after next are fetched, A's in sub-step 0 into the third A
    //         buffer (free since the previous iteration's barrier), B's in sub-step 1, after the barrier,
    //         into the running B buffer: the load path carries the same number of bytes in either sub-step.
    auto substep = [&](auto s_c, auto read_c, auto load_c, auto phase_c) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value;
        constexpr int P0 = PB + (decltype(phase_c)::value ? NM / 8 : 0);   // MFMAs before the first cluster
        constexpr int R = 3 * NM / 4 - P0;
        constexpr bool READ = decltype(read_c)::value, LOAD = decltype(load_c)::value;
        static_assert(!LOAD || READ, "loads go out in iterations that have a successor");
        wait_fragments(s_c);
        AXONN_FENCE();
        mfma_range(s_c, Int<0>{}, Int<PB>{});
        AXONN_FENCE();
        typename OpA::Cursor ca = opa.template cursor<1 - S>(S == 1 ? a1 : a0);
        typename OpB::Cursor cb = opb.template cursor<1 - S>(S == 1 ? b1 : b0);
        if constexpr (READ && S == 1) {
            // the next iteration's panels have landed: every load of this wave but the A loads that
            // sub-step 0 has just issued (loads complete in order) ...
            wait_vmcnt<!LOAD ? 0 : SCHED == 1 ? QLA : SCHED == 2 ? QLB : SCHED == 3 ? NLD / 2 : 0>();
            __builtin_amdgcn_s_barrier();    // ... and of the others; and the running buffers are free
            AXONN_FENCE();
        }
        if constexpr (P0 > PB) {
            mfma_range(s_c, Int<PB>{}, Int<P0>{});
            AXONN_FENCE();
        }
        static_for<NC>([&](auto q_c) __attribute__((always_inline)) {
            constexpr int Q = decltype(q_c)::value;
            if constexpr (READ) read_cluster(q_c, Int<1 - S>{}, ca, cb);
            if constexpr (LOAD && (S == 1 || SCHED != 0)) load_cluster(q_c, s_c, NAB == 3 ? a2 : a0, NBB == 3 ? b2 : b0);
            AXONN_FENCE();
            if constexpr (Q < NC - 1)
                mfma_range(s_c, Int<P0 + Q * R / (NC - 1)>{}, Int<P0 + (Q + 1) * R / (NC - 1)>{});
            else
                mfma_range(s_c, Int<P0 + R>{}, Int<NM>{});
            AXONN_FENCE();
        });
        if constexpr (LOAD) {   // the window moves on behind an operand's last load of the iteration
            if constexpr (SCHED == 1 ? S == 0 : S == 1) opa.advance();
            if constexpr (SCHED == 2 ? S == 0 : S == 1) opb.advance();
        }
        if constexpr (S == 1) {
            // the buffers move up: the one the loads have just gone to (SCHED 0: the running one) comes last
            const uint32_t a = a0, b = b0;
            a0 = a1;
            b0 = b1;
            if constexpr (NAB == 3) {
                a1 = a2;
                a2 = a;
            } else {
                a1 = a;
            }
            if constexpr (NBB == 3) {
                b1 = b2;
                b2 = b;
            } else {
                b1 = b;
            }
        }
    };
    using Yes = std::true_type;
    using No = std::false_type;

    const int KI = ktotal / Cfg::KS;   // at least 2
    // The last sub-step can be taken block row by block row, every finished row converted, staged and
    // stored while the next ones are still being multiplied.  The staging area is the OTHER buffer:
    // every wave released it at the barrier of iteration KI-2 (all fragments of that iteration were in
    // registers by then), and nothing is fetched into it afterwards, so the barrier before the epilogue
    // goes away as well.  Measured on the benchmark's products, three alternating runs each: the TN
    // ones 0.8 % faster (204.6 -> 202.7 us), the NT and NN ones 0.1-0.3 % slower, hence TN only.
    constexpr bool OVERLAP_EPI = !SPLITK && !A_KC && !B_KC;
    auto run = [&](auto phase_c) __attribute__((always_inline)) {
        // fragments of iteration 0, sub-step 0 (inside the phase's own code path: no join between a read and its wait)
        {
            const typename OpA::Cursor ca = opa.template cursor<0>(0u);
            const typename OpB::Cursor cb = opb.template cursor<0>(0u);
            static_for<NC>([&](auto q_c) __attribute__((always_inline)) { read_cluster(q_c, Int<0>{}, ca, cb); });
        }
        for (int it = KI - 2; it > 0; --it) {
            substep(Int<0>{}, Yes{}, Yes{}, phase_c);
            substep(Int<1>{}, Yes{}, Yes{}, phase_c);
        }
        substep(Int<0>{}, Yes{}, No{}, phase_c);   // iteration KI-2: nothing left to fetch
        substep(Int<1>{}, Yes{}, No{}, phase_c);
        substep(Int<0>{}, Yes{}, No{}, phase_c);   // iteration KI-1
        if constexpr (!OVERLAP_EPI) {
            substep(Int<1>{}, No{}, No{}, phase_c);
        } else {
            wait_fragments(Int<1>{});
            AXONN_FENCE();
            static_assert(NW * 16 * TN * 2 <= (int)ABUF, "staging area of the streamed epilogue");
            uint8_t* const epi = smem + (NAB == 3 ? a2 : a1) + wave * (16 * TN * 2);   // the A buffer of the iteration before
            uint16_t* const pc = C + (m0 + wm * TM) * (int64_t)ldc + n0 + wn * TN;
            static_for<MI>([&](auto i_c) __attribute__((always_inline)) {
                constexpr int I = decltype(i_c)::value;
                mfma_range(Int<1>{}, Int<I * NI>{}, Int<(I + 1) * NI>{});
                AXONN_FENCE();
                if constexpr (I > 0) store_block_row16<TN, NI>(acc[I - 1], epi, pc + (int64_t)((I - 1) * 16) * ldc, ldc, lane);
                AXONN_FENCE();
            });
            store_block_row16<TN, NI>(acc[MI - 1], epi, pc + (int64_t)((MI - 1) * 16) * ldc, ldc, lane);
        }
    };
    // With two waves per SIMD the second one (waves 4-7) can issue its clusters an eighth of a sub-step
    // later, so that one wave's reads and loads fall into the other's MFMA runs.  Measured on the
    // benchmark's NT product without split-K: 205 -> 196 us.  It takes a second copy of the loop, and in
    // every other instantiation that copy makes the register allocator spill (TN 199 -> 222 us, NN with two
    // K ranges 210 -> 262), so it is used where it fits only.
    constexpr bool PHASED = NW == 8 && A_KC && B_KC && !SPLITK;
    if constexpr (PHASED) {
        if (wave >= 4) run(Int<1>{});   // wave-uniform; both paths hit the same barriers
        else run(Int<0>{});
    } else {
        run(Int<0>{});
    }
    if constexpr (!OVERLAP_EPI) {
        __syncthreads();   // every wave is done with the buffers before the epilogue reuses LDS
        if constexpr (SPLITK) {
            if (split_k_exchange16<BM, BN, MI, NI>(acc, sk, krange, work.tile_id, tiles_m * tiles_n, wave, lane, t)) return;
        }
        store_tile16<TM, TN, MI, NI>(acc, smem, C + (m0 + wm * TM) * (int64_t)ldc + n0 + wn * TN, ldc, wave, lane);
    }
#undef AXONN_FENCE
}

}  // namespace axonn
