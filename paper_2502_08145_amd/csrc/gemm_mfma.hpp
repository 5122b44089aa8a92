// bf16 x bf16 -> fp32 -> bf16 GEMM tile kernel for gfx950 (CDNA4): one output tile per workgroup
// (or per `splits` workgroups, each over one K range).
//
//   C[M,N] = sum_k a(i,k) b(k,j)      (the local matrix multiply of Algorithm 1 lines 3, 11, 13)
//
// How the kernel is put together, in the order data moves:
//
//  * 4 waves (one per SIMD, 2 x 2) or 8 waves (two per SIMD, 2 x 4) own a BM x BN output tile;
//    the accumulators (up to 256 fp32 per lane) never leave the register file.
//  * K is consumed 32 at a time.  The operand panels of a K-step live in one stage of an LDS ring
//    of NS stages (as many as fit in 160 KB: 5 for the 256x256 tile); panels are fetched NS-2 and
//    NS-1 K-steps ahead of their use.  Global memory goes STRAIGHT into LDS
//    (global_load_lds_dwordx4: 16 bytes per lane, no VGPR staging, no LDS store instruction); the
//    loads of a K-step are spread over the whole step, a few per cluster.
//  * An operand is either "K-contiguous" in global memory (A of NN/NT, B of NT) or
//    "MN-contiguous" (A of TN, B of NN/TN):
//      - K-contiguous panels sit in LDS as rows of 32 k (64 bytes) with the four 16-byte chunks
//        of a row XOR-swizzled by (row>>2)&3, and are read with ds_read_b128: lane l gets, for
//        row l%32, the eight k values 8*(l/32)..+7 that v_mfma_f32_32x32x16_bf16 wants.  Their
//        loads go out in pairs (two K-steps of the same rows back to back) so that both halves of
//        every 128-byte cache line are fetched together.
//      - MN-contiguous panels sit in LDS exactly as in memory, one LDS row per k, with the 16-byte
//        chunks of k-row k XOR-swizzled by 4*(k&3), and are read with the transposing
//        ds_read_b64_tr_b16 (two per fragment).  No register transposes anywhere.
//    Both swizzles make every read conflict-free on the 64-bank LDS, and because a direct load
//    writes 1 KB of consecutive LDS per wave the swizzle is applied by choosing WHICH 16 bytes of
//    global memory each lane fetches.
//  * The main loop is scheduled by hand.  Measurements on MI355X show that one wave per SIMD
//    loses about six matrix-pipe cycles for every interruption of a run of MFMAs, whatever the
//    interruption is, so all non-MFMA work of a half K-step (fragment reads, direct loads) is
//    issued in two clusters, and the loop contains next to no address arithmetic: an LDS address
//    is (precomputed VGPR + stage offset) plus an immediate, a global address a precomputed SGPR
//    base plus one VGPR offset that advances once per K-step.  Loads and LDS reads are inline
//    asm (the compiler would otherwise re-derive addresses with VALU instructions and pick the
//    64-bit-VGPR addressing form); the waits on them are therefore written out by hand too.
//    With two waves per SIMD the second wave's clusters are shifted into the first one's MFMA runs.
//  * One barrier per K-step, placed in the MIDDLE of the step's MFMAs: by then the next stage has
//    landed (vmcnt) and this stage's last fragments are in registers, so the barrier both
//    publishes stage t+1 and releases stage t for refilling.
//  * MFMAs are issued as mfma(Bfrag, Afrag): the 32x32 result block then holds, in lane l, column
//    m = l%32 and FOUR CONSECUTIVE n per accumulator quad, so the epilogue packs 4 bf16 into one
//    8-byte LDS store, transposes the tile through LDS and writes C with 16-byte coalesced
//    stores.  fp32 -> bf16 is round-to-nearest-even, once.
//  * Workgroup ids are remapped so that each of the 8 XCDs (which receive consecutive ids
//    round-robin and have private L2s) works on a compact patch of output tiles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace axonn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int KB = 32;   // k per LDS stage; K must be a multiple of it

template <int V>
using Int = std::integral_constant<int, V>;

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(Int<Is>{}), ...);
}
// f(Int<0>{}), f(Int<1>{}), ... f(Int<N-1>{}): indices usable as template arguments
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Two fp32 -> two bf16 in one word (lo in bits 0..15), round to nearest even; overflow rounds to
// inf, NaN stays NaN.  gfx950 has an instruction for exactly this (v_cvt_pk_bf16_f32), which the
// compiler selects for the vector conversion.
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(size_t)((__attribute__((address_space(3))) const uint8_t*)p);
}

// One wave-level direct load: lane l fetches 16 bytes at base + voff and they land in LDS at
// lds_dst + 16*l (lds_dst and base wave-uniform).  M0 carries the LDS address; the s_nop covers
// the M0-write -> LDS-DMA hazard.  Completion is tracked by vmcnt.  (No immediate offset is used:
// the hardware would add it to the LDS address as well.)
__device__ __forceinline__ void direct_load16(uint32_t lds_dst, const uint8_t* base, uint32_t voff) {
    // wave-uniform by construction; saying so costs nothing where the compiler knows it already and
    // keeps the operand in an SGPR where its analysis gives up
    lds_dst = __builtin_amdgcn_readfirstlane(lds_dst);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(base), "s"(lds_dst) : "memory", "m0");
}
// LDS reads.  An LDS read completes asynchronously and the compiler does not know that: to it the
// asm statement has produced its result at once.  The destination is therefore declared read-write
// ("+v"), which pins a fragment to ONE set of registers for the whole kernel: the compiler can then
// neither rename the destination onto a register that an MFMA issued just before still has to read,
// nor satisfy a later use from a copy made before the data arrived.  (For the same reason the reads
// and the s_waitcnt that covers them always sit in the same straight-line piece of code.)
template <int IMM>
__device__ __forceinline__ void lds_read128(u32x4& dst, uint32_t addr) {
    static_assert(IMM >= 0 && IMM < 65536, "LDS immediate offset is 16 bits");
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "+v"(dst) : "v"(addr), "n"(IMM));
}
template <int IMM>
__device__ __forceinline__ void lds_read64_tr(u32x2& dst, uint32_t addr) {
    static_assert(IMM >= 0 && IMM < 65536, "LDS immediate offset is 16 bits");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "+v"(dst) : "v"(addr), "n"(IMM));
}
// A wave's TM x TN block of bf16 C, staged in LDS at `epi` (rows of TN * 2 bytes, 16-byte chunks
// XOR-swizzled by the row), to global memory in 16-byte coalesced NON-TEMPORAL stores.  C is written
// once and not read again by the kernel; written the ordinary way it displaces operand panels from
// the L2 that other workgroups of the XCD are about to re-read.  Measured in the benchmark's sequence
// of 12 products against ordinary stores: 2.5-5 % less time for outputs of 16-50 MB (most for the
// split-K products), within +-1 % for outputs of 128 MB and more, 1.6 % on the whole step.
template <int TM, int TN>
__device__ __forceinline__ void flush_c_block(const uint8_t* epi, uint16_t* pc, int ldc, int lane) {
    constexpr int CPR = TN / 8;   // 16-byte chunks per row
    constexpr uint32_t CMASK = CPR - 1;
#pragma unroll
    for (int it = 0; it < (TM * CPR) / 64; ++it) {
        const uint32_t idx = it * 64 + lane;
        const uint32_t row = idx / CPR, ch = idx % CPR;
        const u32x4 v = *reinterpret_cast<const u32x4*>(epi + row * (TN * 2) + ((ch ^ (row & CMASK)) << 4));
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(pc + (int64_t)row * ldc + ch * 8));
    }
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// MFMA operand fragment of one 32-row block: eight bf16 per lane.  A b128 read fills it in one go,
// a pair of transposing b64 reads fills its halves.
struct Frag128 {
    u32x4 v;
    __device__ __forceinline__ void clear() { v = u32x4{0, 0, 0, 0}; }
    __device__ __forceinline__ bf16x8 get() const { return __builtin_bit_cast(bf16x8, v); }
};
struct Frag64x2 {
    u32x2 lo, hi;
    __device__ __forceinline__ void clear() { lo = hi = u32x2{0, 0}; }
    __device__ __forceinline__ bf16x8 get() const {
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3));
    }
};
// All LDS reads issued so far have landed.  The fragment registers are made to depend on the wait
// so that no MFMA reading them can be scheduled above it.
template <int N>
__device__ __forceinline__ void tie_to_lds_wait(Frag128* f) {
    static_assert(N == 1 || N == 2 || N == 4, "1, 2 or 4 blocks a side");
    if constexpr (N == 4)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].v), "+v"(f[1].v), "+v"(f[2].v), "+v"(f[3].v)::"memory");
    else if constexpr (N == 2)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].v), "+v"(f[1].v)::"memory");
    else
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].v)::"memory");
}
template <int N>
__device__ __forceinline__ void tie_to_lds_wait(Frag64x2* f) {
    static_assert(N == 1 || N == 2 || N == 4, "1, 2 or 4 blocks a side");
    if constexpr (N == 4)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi), "+v"(f[2].lo), "+v"(f[2].hi),
                       "+v"(f[3].lo), "+v"(f[3].hi)::"memory");
    else if constexpr (N == 2)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi)::"memory");
    else
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi)::"memory");
}

// ------------------------------------------------------------------------------------------------
// Operand policies.  ROWS = tile extent along m (or n); REGION = byte offset of the operand's
// panel inside a stage.  Each policy gives
//   init(...)                  per-lane / per-wave constants
//   issue<C, AHEAD>(stage_off) the C-th of QL direct loads of this wave into the stage at stage_off,
//                              for the K-step AHEAD (0/1) steps past the global window
//   advance()                  move the global window one K-step on
//   PAIR                       see below: the operand wants its loads issued two K-steps at a time
//   cursor(stage_off)          the VGPR addresses for reading that stage (made once per K-step)
//   read<I, S>(frag, cursor)   fragment of 32-row block I, k16 substep S (0/1)
// The stage offset is the only run-time part of an LDS address; everything else is an immediate.
// ------------------------------------------------------------------------------------------------
// SWZ: the four 16-byte chunks of LDS row r are XOR-swizzled by (r >> SWZ) & 3.  ds_read_b128 runs at
// full rate (256 B/clk) only if the swizzle suits the fragment shape: 2 for the 32-row fragments of
// the 32x32x16 MFMA (lane l: row l%32, chunk l/32), 1 for the 16-row fragments of the 16x16x32 MFMA
// (lane l: row l%16, chunk l/16); the other way round, or without swizzle, it runs at half rate
// (measured with a read-only microbenchmark: 570 against 305 bytes/ns per CU).
template <int ROWS, int REGION, int NW, int NB_, int SWZ = 2>
struct OperandKContig {   // global P[row * ld + k]
    static_assert(SWZ == 1 || SWZ == 2, "swizzle by (row>>1)&3 or (row>>2)&3");
    static constexpr int QL = ROWS / 16 / NW;  // a load covers 16 rows x 64 B
    static constexpr int NB = NB_;             // 32-row blocks per wave tile
    static_assert(QL >= 1, "at least one load per wave and stage");
    // A row's 32 k of one K-step are half a 128-byte cache line.  Fetching the two halves a K-step
    // apart costs a second trip to L2 (the L1 has turned over by then); fetched back to back the
    // second one hits in L1.  So the loads of such an operand go out in pairs: the same 16 rows for
    // two consecutive K-steps, into two stages.  A wave's QL row groups are served alternately:
    // the even ones in even K-steps, the odd ones in odd K-steps (needs QL even); which of the two
    // is a run-time state (row offset folded into voff, LDS offset in lds_par), so that the K loop
    // is one piece of code.
    static constexpr bool PAIR = QL % 2 == 0;
    static constexpr int NBASE = PAIR ? QL / 2 : QL;   // row groups with a base pointer of their own
    struct Cursor {
        uint32_t a[2];   // [substep]
    };
    const uint8_t* base[NBASE];                  // uniform: first row of load c (PAIR: of load 2c), k = 0
    uint32_t lds_dst[NBASE];                  // uniform: its destination inside stage 0
    uint32_t voff[2];                          // per lane: row-in-load * ld + fetched chunk * 16 + window
                                               // (+ 16 rows when the odd groups are served); [1]: one K-step on
    uint32_t lds_par;                          // uniform, PAIR: 1024 when the odd groups are served
    uint32_t step_add;                         // uniform, PAIR: what advance() adds to voff
    uint32_t raddr[2];                         // [substep]: read address of block 0 in stage 0
    uint32_t raddr16;                          // the same for 16-row blocks read 32 k at a time

    // first_step_odd: the first (virtual) K-step of the load schedule serves the odd row groups
    __device__ __forceinline__ void init(const uint16_t* P, int64_t row0, uint32_t ld_bytes, int lane, int wave,
                                         uint32_t lds0, int wave_row_base, bool first_step_odd) {
        const uint8_t* origin = reinterpret_cast<const uint8_t*>(P) + (size_t)row0 * ld_bytes;
        constexpr int STRIDE = PAIR ? 2 : 1;
#pragma unroll
        for (int c = 0; c < NBASE; ++c) {
            base[c] = origin + (size_t)(16 * (wave * QL + STRIDE * c)) * ld_bytes;
            lds_dst[c] = lds0 + REGION + (wave * QL + STRIDE * c) * 1024;
        }
        // lane -> LDS slot (row = lane>>2, slot = lane&3); that slot holds chunk slot ^ ((row>>SWZ)&3)
        voff[0] = (lane >> 2) * ld_bytes + (((lane & 3) ^ ((lane >> (2 + SWZ)) & 3)) << 4);
        const uint32_t group_bytes = 16 * ld_bytes;
        lds_par = 0;
        step_add = KB * 2 + group_bytes;
        if (PAIR && first_step_odd) {
            voff[0] += group_bytes;
            lds_par = 1024;
            step_add = KB * 2 - group_bytes;
        }
        voff[1] = voff[0] + KB * 2;
        // reader: row = wave_row_base + 32*I + lane%32 ((row>>SWZ)&3 does not depend on I),
        // chunk = 2*S + lane/32
        const uint32_t row = wave_row_base + (lane & 31);
        const uint32_t a0 = lds0 + REGION + row * 64 + (((lane >> 5) ^ ((row >> SWZ) & 3)) << 4);
        raddr[0] = a0;
        raddr[1] = a0 ^ 32;
        // 16x16x32 reader: row = wave_row_base + 16*I + lane%16 ((row>>SWZ)&3 = (lane>>SWZ)&3 for every I),
        // chunk = lane/16
        raddr16 = lds0 + REGION + (wave_row_base + (lane & 15)) * 64 + ((((lane >> 4) & 3) ^ ((lane >> SWZ) & 3)) << 4);
    }
    // Load number C of the current K-step (PAIR: for pair C of the row groups now served), for the
    // K-step AHEAD past the window, into the stage at stage_off.
    template <int C, int AHEAD>
    __device__ __forceinline__ void issue(uint32_t stage_off) const {
        static_assert(C < NBASE && (AHEAD == 0 || PAIR), "no such load");
        if constexpr (PAIR)
            direct_load16(lds_dst[C] + stage_off + lds_par, base[C], voff[AHEAD]);
        else
            direct_load16(lds_dst[C] + stage_off, base[C], voff[0]);
    }
    // next K-step: window one step on and, PAIR, the other row groups
    __device__ __forceinline__ void advance() {
        if constexpr (PAIR) {
            voff[0] += step_add;
            voff[1] += step_add;
            step_add = 4 * KB - step_add;
            lds_par ^= 1024;
        } else {
            voff[0] += KB * 2;
        }
    }
    // PAIR: the other row groups, same window
    __device__ __forceinline__ void flip() {
        static_assert(PAIR, "paired operands only");
        voff[0] += step_add - KB * 2;
        voff[1] += step_add - KB * 2;
        step_add = 4 * KB - step_add;
        lds_par ^= 1024;
    }
    __device__ __forceinline__ Cursor cursor(uint32_t stage_off) const {
        return Cursor{{raddr[0] + stage_off, raddr[1] + stage_off}};
    }
    using Frag = Frag128;
    template <int I, int S>
    __device__ __forceinline__ void read(Frag& f, const Cursor& c) const {
        lds_read128<I * 2048>(f.v, c.a[S]);
    }
    // fragments of v_mfma_f32_16x16x32_bf16: 16-row block I, all 32 k of the stage (lane l: row l%16,
    // k = 8*(l/16)..+7)
    struct Cursor16 {
        uint32_t a;
    };
    __device__ __forceinline__ Cursor16 cursor16(uint32_t stage_off) const { return Cursor16{raddr16 + stage_off}; }
    template <int I>
    __device__ __forceinline__ void read16(Frag& f, const Cursor16& c) const {
        lds_read128<I * 1024>(f.v, c.a);
    }
};

// TR16: layout for the 16x16x32 fragments.  A transposing read serves its four 16-lane groups (k
// blocks of 8) two at a time, provided the two groups of a pair fall into different halves of the
// 64 banks and the four k-rows of a group into one contiguous 128 bytes; with the 32x32x16 layout
// (chunks swizzled by 4*(k&3)) every group lands on the same banks and the read runs at half rate
// (measured with a read-only microbenchmark: 296 against 520 bytes/ns per CU).  So chunk c of k-row
// k sits at position c ^ 2*(k&3) ^ 8*((k>>3)&1).  The swizzle now touches the chunk bits that
// number a wave's 16-row blocks, so every block has an address register of its own.
template <int ROWS, int REGION, int NW, int NB_, bool TR16 = false>
struct OperandMNContig {   // global P[k * ld + row]
    static constexpr int ROWB = ROWS * 2;              // bytes per k-row in LDS
    static constexpr int KR = 1024 / ROWB;             // k-rows per load: 2 (256 rows) or 4 (128 rows)
    static constexpr int QL = KB / KR / NW;
    static constexpr int NB = NB_;
    static_assert(QL >= 1 && (KR == 4 || QL % 2 == 0), "loads per wave: whole, and even when a load holds two k-rows");
    static constexpr int CPR = ROWB / 16;              // 16-byte chunks per k-row
    static_assert(ROWS == 128 || ROWS == 256, "tile extents are 128 or 256");
    struct Cursor {
        uint32_t a[NB];
    };
    const uint8_t* base;       // uniform: k-row 0 of the wave's first load; the K window moves here
    uint32_t voff[QL];         // per lane and load: k-row inside the wave's share * ld + fetched chunk * 16
    size_t kstep_bytes;        // uniform: KB k-rows
    uint32_t lds_dst[QL];
    uint32_t raddr[NB];        // [block]: read address in stage 0 for substep 0, first four k
    static constexpr int NA16 = TR16 ? 2 * NB : NB;
    uint32_t raddr16[NA16];    // 16x16x32 fragments: [pair of 16-row blocks], TR16: [16-row block]

    __device__ __forceinline__ void init(const uint16_t* P, int64_t row0, uint32_t ld_bytes, int lane, int wave,
                                         uint32_t lds0, int wave_row_base, bool /*first_step_odd*/) {
        const uint8_t* origin = reinterpret_cast<const uint8_t*>(P) + (size_t)row0 * 2;
        base = origin + (size_t)(KR * QL * wave) * ld_bytes;
#pragma unroll
        for (int c = 0; c < QL; ++c) lds_dst[c] = lds0 + REGION + (wave * QL + c) * 1024;   // load c carries k-rows KR*(wave*QL + c) ..
        // lane -> (k-row kr of the load, LDS chunk position lane % CPR); that position holds chunk
        // pos ^ 4*(k&3).  k = KR*q + kr: for KR == 4, k&3 = kr; for KR == 2, k&3 = 2*(c&1) + kr
        // (wave*QL is even).
        const uint32_t kr = lane / CPR, pos = lane % CPR;
        const uint32_t k3_even = kr, k3_odd = (KR == 2) ? 2 + kr : kr;
        static_assert(KR * QL <= 8, "a wave's loads stay inside one block of eight k-rows");
        const uint32_t kb = ((uint32_t)(KR * QL * wave) >> 3) & 1u;   // (k>>3)&1, the same for all loads of a wave
#pragma unroll
        for (int c = 0; c < QL; ++c) {
            const uint32_t k3 = (c & 1) ? k3_odd : k3_even;
            const uint32_t swz = TR16 ? (2 * k3) ^ (8 * kb) : 4 * k3;
            voff[c] = (uint32_t)(KR * c + kr) * ld_bytes + ((pos ^ swz) << 4);
        }
        kstep_bytes = (size_t)KB * ld_bytes;
        // reader (transposing read, 16-lane groups): group g = lane/16 covers m-half g&1 and
        // k-half g>>1; lane s of a group addresses k-row (s>>2) and 4 consecutive m at 4*(s&3).
        const uint32_t sl = lane & 15, g = lane >> 4, kq = sl >> 2;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const uint32_t m = wave_row_base + i * 32 + 16 * (g & 1) + 4 * (sl & 3);
            raddr[i] = lds0 + REGION + (kq + 8 * (g >> 1)) * ROWB + (((m >> 3) ^ (4 * kq)) << 4) + (m & 4) * 2;
        }
        // 16x16x32 reader: group g covers k = 8g..8g+7 (two reads of four k-rows) for the 16 rows of a
        // block; lane s of a group addresses k-row (s>>2) and 4 consecutive m at 4*(s&3).  Blocks 2p
        // and 2p+1 differ by 32 bytes (chunk bit 1, which neither the swizzle nor a carry touches).
#pragma unroll
        for (int p = 0; p < NA16; ++p) {
            if constexpr (TR16) {
                const uint32_t m = wave_row_base + p * 16 + 4 * (sl & 3);
                raddr16[p] = lds0 + REGION + (kq + 8 * g) * ROWB + (((m >> 3) ^ (2 * kq) ^ (8 * (g & 1))) << 4) + (m & 4) * 2;
            } else {
                const uint32_t m = wave_row_base + p * 32 + 4 * (sl & 3);
                raddr16[p] = lds0 + REGION + (kq + 8 * g) * ROWB + (((m >> 3) ^ (4 * kq)) << 4) + (m & 4) * 2;
            }
        }
    }
    static constexpr bool PAIR = false;   // a load already covers whole cache lines
    static constexpr int NBASE = QL;
    template <int C, int AHEAD>
    __device__ __forceinline__ void issue(uint32_t stage_off) const {
        static_assert(AHEAD == 0, "loaded one K-step at a time");
        direct_load16(lds_dst[C] + stage_off, base, voff[C]);
    }
    // One K-step on.  The window moves in the (64-bit, scalar) base pointers, not in the 32-bit
    // per-lane offsets: a panel of more than 4 GB (K * ld * 2 bytes) would wrap those.
    __device__ __forceinline__ void advance() { base += kstep_bytes; }
    __device__ __forceinline__ Cursor cursor(uint32_t stage_off) const {
        Cursor c;
#pragma unroll
        for (int i = 0; i < NB; ++i) c.a[i] = raddr[i] + stage_off;
        return c;
    }
    using Frag = Frag64x2;
    template <int I, int S>
    __device__ __forceinline__ void read(Frag& f, const Cursor& c) const {
        static_assert(!TR16, "the 32x32x16 reader goes with the 32x32x16 layout");
        // k = 16*S + 8*(lane/32) + 0..3 and + 4..7
        lds_read64_tr<(16 * S) * ROWB>(f.lo, c.a[I]);
        lds_read64_tr<(16 * S + 4) * ROWB>(f.hi, c.a[I]);
    }
    struct Cursor16 {
        uint32_t a[NA16];
    };
    __device__ __forceinline__ Cursor16 cursor16(uint32_t stage_off) const {
        Cursor16 c;
#pragma unroll
        for (int p = 0; p < NA16; ++p) c.a[p] = raddr16[p] + stage_off;
        return c;
    }
    template <int I>
    __device__ __forceinline__ void read16(Frag& f, const Cursor16& c) const {
        if constexpr (TR16) {
            lds_read64_tr<0>(f.lo, c.a[I]);
            lds_read64_tr<4 * ROWB>(f.hi, c.a[I]);
        } else {
            lds_read64_tr<(I & 1) * 32>(f.lo, c.a[I / 2]);
            lds_read64_tr<(I & 1) * 32 + 4 * ROWB>(f.hi, c.a[I / 2]);
        }
    }
};

// ------------------------------------------------------------------------------------------------
// Split-K: when an output has too few tiles to occupy the chip, `splits` workgroups share a tile,
// each reducing one contiguous K range.  The workgroups of ranges 1..splits-1 ("writers") park their
// fp32 accumulators in a scratch slot and raise a flag; the workgroup of range 0 ("reader") adds the
// slots to its own accumulators in range order and writes C, so the result does not depend on timing.
// Writers never wait and have the lower workgroup ids on every XCD, so they are dispatched before the
// readers that depend on them and a reader's wait always ends; the wait is bounded anyway.
struct SplitK {
    float* partials;      // [(splits-1) * tiles] slots of BM*BN floats, in accumulator order
    uint32_t* flags;      // [(splits-1) * tiles]; a slot is valid when its flag equals `epoch`; the reader resets it to 0
    uint32_t* timeouts;   // incremented when a reader gives up waiting (never, unless a writer died)
    uint32_t epoch;       // non-zero, differs from launch to launch: a flag left behind by a launch that died is never valid
    int splits;           // 1: no split
};
constexpr uint32_t kSplitSpinLimit = 1u << 19;   // x ~3 us per probe
constexpr int kSplitRangePerXcdK = 32768;        // four K ranges: from this K on, one range per pair of XCDs

// Workgroup -> output tile and K range.  The hardware hands workgroup b to XCD b % 8, in order of b
// on each XCD, and every XCD has a private L2: ids are remapped so that an XCD works on a contiguous
// chunk of the tile sequence, and tiles are then grouped `group_m` along m, which makes the tiles
// running side by side behind one L2 a compact patch of the output (they share operand panels).
// Split-K: the workgroups of a tile sit on the same XCD, last K range first (writers get the lower
// ids) -- except with four ranges of a large tile at long K, where XCDs 0-1 take the last K range,
// ..., XCDs 6-7 range 0, each a contiguous chunk of the tiles, so the 32 workgroups that share an L2
// read the same K slices (with all four ranges of a tile on one XCD they would share a quarter as
// much; measured 17-20 % faster at K = 65536 for NN and NT).  The readers then sit on two XCDs only,
// which makes the exchange slower by some 10 us: not for short K.  Writers keep the lower ids there
// too (same pid >> 3, lower XCD).
struct TileWork {
    int tile_id;          // index into the tile sequence (= split-K slot index within a range)
    int tile_m, tile_n;
    int krange, ktotal;   // this workgroup's K range and its length
};
template <bool SPLITK, bool LARGE_TILE>
__device__ __forceinline__ TileWork map_workgroup(int pid, int nwg, int K, int tiles_m, int tiles_n, int group_m,
                                                  const SplitK& sk) {
    TileWork w;
    w.krange = 0;
    w.ktotal = K;
    if constexpr (SPLITK) {
        const int splits = sk.splits, tiles = tiles_m * tiles_n;
        if (LARGE_TILE && splits == 4 && (nwg & 7) == 0 && K >= kSplitRangePerXcdK) {
            const int x = pid & 7, q = pid >> 3, tp = tiles >> 1;
            w.krange = 3 - (x >> 1);
            pid = (x & 1) * tp + q;
        } else if (nwg % (8 * splits) == 0) {
            const int tp = (nwg >> 3) / splits, li = pid >> 3;
            w.krange = splits - 1 - li / tp;
            pid = (pid & 7) * tp + li % tp;
        } else {
            w.krange = splits - 1 - pid / tiles;
            pid = pid % tiles;
        }
        w.ktotal = K / splits;
    } else {
        if ((nwg & 7) == 0) pid = (pid & 7) * (nwg >> 3) + (pid >> 3);
    }
    w.tile_id = pid;
    const int group_sz = group_m * tiles_n;
    const int group = pid / group_sz;
    const int first_m = group * group_m;
    const int gm = min(tiles_m - first_m, group_m);
    const int in_group = pid - group * group_sz;
    w.tile_m = first_m + in_group % gm;
    w.tile_n = in_group / gm;
    return w;
}

// ------------------------------------------------------------------------------------------------
// NS = number of LDS stages: as many as fit (160 KB per CU; the 128x128 tile takes 80 KB so that
// two workgroups share a CU).  WM x WN waves: 2 x 2 (one wave per SIMD) or 2 x 4 (two).
template <int BM, int BN, int WM, int WN>
struct TileCfg {
    static constexpr int NW = WM * WN;
    static constexpr int NT = 64 * NW;
    static constexpr int TM = BM / WM, TN = BN / WN;        // wave tile
    static constexpr int MI = TM / 32, NI = TN / 32;        // 32x32 blocks per wave tile
    static constexpr int STAGE_BYTES = (BM + BN) * KB * 2;  // A panel then B panel
    static constexpr int NS = (BM + BN == 512) ? 5 : (BM + BN == 384) ? 6 : 5;
    static constexpr int RING_BYTES = NS * STAGE_BYTES;
    static constexpr int EPI_BYTES = BM * BN * 2;
    static constexpr int LDS_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
    static constexpr int MIN_K = KB * (NS - 1);             // the prologue fills NS-1 stages
    static_assert((BM == 128 || BM == 256) && (BN == 128 || BN == 256), "tile extents are 128 or 256");
    static_assert(WM == 2 && (WN == 2 || WN == 4), "4 or 8 waves");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
};

// Book-keeping of the direct loads in flight (vmcnt counts them in issue order).  A K-step is of
// kind 2 (issues all NL loads of a wave), 1 (only the first halves of paired operands' pairs) or 0
// (none); the steps after the last full one are "tail" steps 0, 1, ...; steps before it (negative
// index) are full.  At the barrier in the middle of a step the loads of the last NS-LAG steps and
// of the step's own first half (operand A) may still be in flight.
template <int QA, int QB, bool PAIR_A, bool PAIR_B, int NS>
struct LoadPlan {
    static constexpr int NL = QA + QB;
    static constexpr bool ANY_PAIR = PAIR_A || PAIR_B;
    static constexpr int LAG = ANY_PAIR ? 4 : 3;
    static_assert(NS >= LAG, "ring too short");
    static constexpr int issued(int kind) {
        return kind == 2 ? NL : kind == 1 ? (PAIR_A ? QA / 2 : 0) + (PAIR_B ? QB / 2 : 0) : 0;
    }
    static constexpr int issued_first_half(int kind) { return kind == 2 ? QA : kind == 1 ? (PAIR_A ? QA / 2 : 0) : 0; }
    static constexpr int tail_kind(int j) { return j < 0 ? 2 : (ANY_PAIR && j == 0) ? 1 : 0; }
    static constexpr int tail_vm(int j) {
        int n = issued_first_half(tail_kind(j));
        for (int s = j - (NS - LAG); s < j; ++s) n += issued(tail_kind(s));
        return n;
    }
};

// Requires M % BM == 0, N % BN == 0, K % 32 == 0, K >= TileCfg::MIN_K (checked on the host).
// With SPLITK the grid holds sk.splits workgroups per tile and additionally (K / sk.splits) % 32 == 0,
// K / sk.splits >= TileCfg::MIN_K.
template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, bool SPLITK>
__global__ __launch_bounds__(64 * WM * WN) void gemm_tile_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
    int K, int lda, int ldb, int ldc, int tiles_m, int tiles_n, int group_m, SplitK sk) {
    using Cfg = TileCfg<BM, BN, WM, WN>;
    constexpr int NW = Cfg::NW;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, MI = Cfg::MI, NI = Cfg::NI, NS = Cfg::NS;
    constexpr uint32_t SB = Cfg::STAGE_BYTES, RING = Cfg::RING_BYTES;
    using OpA = typename std::conditional<A_KC, OperandKContig<BM, 0, NW, MI>, OperandMNContig<BM, 0, NW, MI>>::type;
    using OpB = typename std::conditional<B_KC, OperandKContig<BN, BM * KB * 2, NW, NI>,
                                          OperandMNContig<BN, BM * KB * 2, NW, NI>>::type;
    constexpr int QA = OpA::QL, QB = OpB::QL, NL = QA + QB;   // direct loads per wave per stage
    constexpr int NM = MI * NI;                                // MFMAs per half K-step
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- workgroup -> output tile and K range ------------------------------------------------
    const TileWork work = map_workgroup<SPLITK, BM * BN == 256 * 256>(blockIdx.x, gridDim.x, K, tiles_m, tiles_n, group_m, sk);
    const int tile_id = work.tile_id, tile_m = work.tile_m, tile_n = work.tile_n, krange = work.krange, ktotal = work.ktotal;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

    const uint32_t lds0 = lds_address(smem);
    OpA opa;
    OpB opb;
    const int64_t k0 = (int64_t)krange * ktotal;
    // the load schedule starts NS-1 K-steps before K-step 0 (see "direct loads" below)
    constexpr bool FIRST_ODD = (NS - 1) % 2 == 1;
    opa.init(A + (A_KC ? k0 : k0 * lda), m0, 2u * (uint32_t)lda, lane, wave, lds0, wm * TM, FIRST_ODD);
    opb.init(B + (B_KC ? k0 : k0 * ldb), n0, 2u * (uint32_t)ldb, lane, wave, lds0, wn * TN, FIRST_ODD);

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // fragment double buffer: [k16 substep parity][block]; cleared once because the LDS reads take
    // them as read-write operands
    typename OpA::Frag fa[2][MI];
    typename OpB::Frag fb[2][NI];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[u][i].clear();
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[u][j].clear();
    }

    // Nothing may be scheduled across this point (keeps the hand-made instruction order).
#define AXONN_FENCE() __builtin_amdgcn_sched_barrier(0)
    // MFMA number IDX (i-major) of a half K-step, on fragment buffer BUF.
    auto mfma = [&](auto buf_c, auto idx_c) __attribute__((always_inline)) {
        constexpr int BUF = decltype(buf_c)::value, I = decltype(idx_c)::value / NI, J = decltype(idx_c)::value % NI;
        acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[BUF][J].get(), fa[BUF][I].get(), acc[I][J], 0, 0, 0);
    };
    auto mfma_range = [&](auto buf_c, auto lo_c, auto hi_c) __attribute__((always_inline)) {
        constexpr int LO = decltype(lo_c)::value, HI = decltype(hi_c)::value;
        static_for<HI - LO>([&](auto d) __attribute__((always_inline)) { mfma(buf_c, Int<LO + decltype(d)::value>{}); });
    };
    auto wait_fragments = [&](auto buf_c) __attribute__((always_inline)) {
        constexpr int BUF = decltype(buf_c)::value;
        tie_to_lds_wait<MI>(fa[BUF]);
        tie_to_lds_wait<NI>(fb[BUF]);
    };
    // Cluster HALF (0/1) of the fragment reads of substep S through the given cursors into buffer BUF:
    // the MI + NI blocks (A first) are split evenly over the two clusters.  The buffer being filled
    // was last read by MFMAs of the previous half K-step, all issued before this half began.
    auto read_cluster = [&](auto half_c, auto s_c, auto buf_c, const typename OpA::Cursor& ca,
                            const typename OpB::Cursor& cb) __attribute__((always_inline)) {
        constexpr int H = decltype(half_c)::value, S = decltype(s_c)::value, BUF = decltype(buf_c)::value;
        constexpr int NBLK = MI + NI, FIRST = H == 0 ? 0 : NBLK / 2, LAST = H == 0 ? NBLK / 2 : NBLK;
        static_for<LAST - FIRST>([&](auto d) __attribute__((always_inline)) {
            constexpr int Q = FIRST + decltype(d)::value;
            if constexpr (Q < MI)
                opa.template read<Q, S>(fa[BUF][Q], ca);
            else
                opb.template read<Q - MI, S>(fb[BUF][Q - MI], cb);
        });
    };
    // ---- direct loads -----------------------------------------------------------------------
    // During K-step t a wave fetches, per operand, QL loads:
    //   plain operand   all its loads of K-step t+NS-1, into the stage K-step t-1 used (stage "far");
    //   paired operand  half its row groups (even ones if t is even, else the odd ones) for the TWO
    //                   K-steps t+NS-2 and t+NS-1, back to back, into the stages "near" (the one
    //                   K-step t-2 used) and "far".
    // Either way a stage is refilled only after the barrier that ended its last use, every K-step
    // issues the same NL loads, and K-step u is complete once the loads of step u-NS+1 (plain) or
    // u-NS+2 (any operand paired) are.  KIND: 2 = all of the above, 1 = K-step t+NS-1 no longer
    // exists (a paired operand still fetches its half of t+NS-2), 0 = nothing.
    auto issue_loads = [&](auto op_c, auto kind_c, auto half_c, uint32_t st_near, uint32_t st_far) __attribute__((always_inline)) {
        constexpr bool IS_A = decltype(op_c)::value == 0;
        constexpr int KIND = decltype(kind_c)::value, H = decltype(half_c)::value;
        using Op = typename std::conditional<IS_A, OpA, OpB>::type;
        auto& op = [&]() __attribute__((always_inline)) -> auto& { if constexpr (IS_A) return opa; else return opb; }();
        constexpr int NB = Op::NBASE, FIRST = H == 0 ? 0 : (NB + 1) / 2, LAST = H == 0 ? (NB + 1) / 2 : NB;
        static_for<LAST - FIRST>([&](auto d) __attribute__((always_inline)) {
            constexpr int C = FIRST + decltype(d)::value;
            if constexpr (Op::PAIR) {
                if constexpr (KIND >= 1) op.template issue<C, 0>(st_near);
                if constexpr (KIND == 2) op.template issue<C, 1>(st_far);
            } else {
                if constexpr (KIND == 2) op.template issue<C, 0>(st_far);
            }
        });
    };
    using Plan = LoadPlan<QA, QB, OpA::PAIR, OpB::PAIR, NS>;
    constexpr int LAG = Plan::LAG;
    auto next_stage = [&](uint32_t off) __attribute__((always_inline)) -> uint32_t { return off + SB == RING ? 0u : off + SB; };

    // ---- prologue: the loads "steps -(NS-1) .. -1" would have issued; K-step 0 visible ----------
    static_for<NS - 1>([&](auto v) __attribute__((always_inline)) {
        constexpr int T = decltype(v)::value - (NS - 1);          // virtual step
        constexpr uint32_t FAR = (T + NS - 1) * SB;               // stage of K-step T+NS-1
        static_for<2>([&](auto op_c) __attribute__((always_inline)) {
            constexpr bool IS_A = decltype(op_c)::value == 0;
            using Op = typename std::conditional<IS_A, OpA, OpB>::type;
            auto& op = [&]() __attribute__((always_inline)) -> auto& { if constexpr (IS_A) return opa; else return opb; }();
            if constexpr (Op::PAIR && T == -(NS - 1)) {
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
    wait_vmcnt<(NS - LAG + 1) * NL>();
    __builtin_amdgcn_s_barrier();
    AXONN_FENCE();
    uint32_t st_cur = 0, st_next = SB;
    uint32_t st_near = (NS - 2) * SB, st_far = (NS - 1) * SB;   // stages of K-steps t+NS-2 and t+NS-1
    // read cursors of the current stage; the ones of the next stage are made in the second half of
    // a step and become the current ones when the step ends
    typename OpA::Cursor ca = opa.cursor(st_cur);
    typename OpB::Cursor cb = opb.cursor(st_cur);

    // ---- one K-step on the stage at st_cur ---------------------------------------------------
    //   KIND: what it fetches (see above).
    //   NEXT: a following K-step exists.
    //   VM:   direct loads that may still be in flight at the barrier (everything older has
    //         landed, in particular the whole of K-step t+1).
    //   PHASE: where the two clusters of a half sit among its NM MFMAs.  With two waves per SIMD the
    //         second wave of each SIMD (waves 4..7) uses phase 1, so that one wave's clusters fall
    //         into the other's runs of MFMAs and the matrix pipe always has work queued.
    auto step = [&](auto phase_c, auto kind_c, auto next_c, auto vm_c) __attribute__((always_inline)) {
        constexpr bool NEXT = decltype(next_c)::value;
        constexpr int VM = decltype(vm_c)::value, KIND = decltype(kind_c)::value;
        constexpr int P0 = decltype(phase_c)::value == 0 ? 1 : NM / 4 + 1;        // MFMAs before cluster 0
        constexpr int P1 = decltype(phase_c)::value == 0 ? NM / 2 + 1 : NM / 4 + NM / 2 + 1;   // ... cluster 1
        // first half: MFMAs of substep 0 (buffer 0); substep-1 fragments into buffer 1
        wait_fragments(Int<0>{});
        AXONN_FENCE();
        mfma_range(Int<0>{}, Int<0>{}, Int<P0>{});
        AXONN_FENCE();
        read_cluster(Int<0>{}, Int<1>{}, Int<1>{}, ca, cb);
        issue_loads(Int<0>{}, kind_c, Int<0>{}, st_near, st_far);
        AXONN_FENCE();
        mfma_range(Int<0>{}, Int<P0>{}, Int<P1>{});
        AXONN_FENCE();
        read_cluster(Int<1>{}, Int<1>{}, Int<1>{}, ca, cb);
        issue_loads(Int<0>{}, kind_c, Int<1>{}, st_near, st_far);
        AXONN_FENCE();
        mfma_range(Int<0>{}, Int<P1>{}, Int<NM>{});
        AXONN_FENCE();
        // middle: the last fragments of this stage are in registers and K-step t+1 has landed
        wait_fragments(Int<1>{});
        if constexpr (NEXT) {
            wait_vmcnt<VM>();
            __builtin_amdgcn_s_barrier();
        }
        AXONN_FENCE();
        // second half: MFMAs of substep 1 (buffer 1); first fragments of K-step t+1 into buffer 0
        mfma_range(Int<1>{}, Int<0>{}, Int<P0>{});
        AXONN_FENCE();
        if constexpr (NEXT) {
            ca = opa.cursor(st_next);
            cb = opb.cursor(st_next);
            read_cluster(Int<0>{}, Int<0>{}, Int<0>{}, ca, cb);
        }
        issue_loads(Int<1>{}, kind_c, Int<0>{}, st_near, st_far);
        AXONN_FENCE();
        mfma_range(Int<1>{}, Int<P0>{}, Int<P1>{});
        AXONN_FENCE();
        if constexpr (NEXT) read_cluster(Int<1>{}, Int<0>{}, Int<0>{}, ca, cb);
        issue_loads(Int<1>{}, kind_c, Int<1>{}, st_near, st_far);
        if constexpr (KIND == 2) {
            opa.advance();
            opb.advance();
        }
        AXONN_FENCE();
        mfma_range(Int<1>{}, Int<P1>{}, Int<NM>{});
        AXONN_FENCE();
        st_near = st_far;
        st_far = st_cur;   // the stage just finished is the last one of the ring to be refilled
        st_cur = st_next;
        st_next = next_stage(st_next);
    };
    using Yes = std::true_type;

    // After KT-NS+1 full steps come the steps that fetch less: one of kind 1 if an operand is
    // paired (K-step KT-1 still lacks that operand's other half), then kind 0 to the end.
    constexpr int NTAIL = NS - 1;
    const int KT = ktotal / KB;   // at least NS - 1
    auto main_loop = [&](auto phase_c) __attribute__((always_inline)) {
        // The first fragments are fetched here, inside the phase's own code path: an LDS read is
        // asynchronous and the compiler does not know it, so between a read and the wait that
        // covers it there must be no point (such as a branch join) where it could copy the
        // destination registers.
        read_cluster(Int<0>{}, Int<0>{}, Int<0>{}, ca, cb);
        read_cluster(Int<1>{}, Int<0>{}, Int<0>{}, ca, cb);
        constexpr int VM_FULL = Plan::tail_vm(-1);
        for (int kt = KT - NTAIL; kt > 0; --kt) step(phase_c, Int<2>{}, Yes{}, Int<VM_FULL>{});
        static_for<NTAIL>([&](auto j_c) __attribute__((always_inline)) {
            constexpr int J = decltype(j_c)::value;
            step(phase_c, Int<Plan::tail_kind(J)>{}, std::integral_constant<bool, (J + 1 < NTAIL)>{},
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

    // ---- split-K exchange: slot element ((wave*MI*NI + i*NI + j)*4 + g)*64 + lane, 16 bytes each ---
    if constexpr (SPLITK) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const int tiles = tiles_m * tiles_n;
        const size_t in_slot = (size_t)wave * (MI * NI * 4 * 64) + lane;
        if (krange != 0) {
            const size_t slot = (size_t)(krange - 1) * tiles + tile_id;
            f32x4* dst = reinterpret_cast<f32x4*>(sk.partials) + slot * (BM * BN / 4) + in_slot;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        dst[((i * NI + j) * 4 + g) * 64] = f32x4{acc[i][j][4 * g], acc[i][j][4 * g + 1],
                                                                 acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
            // Cache maintenance is dear on a chip of eight private L2s (a device-scope release writes
            // the L2 back, an acquire invalidates it), so each workgroup does it once: the barrier
            // orders every thread's stores before thread 0's release, and thread 0's acquire before
            // every thread's loads.
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
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // no stale cached copy of the slot
            }
            __syncthreads();
            const f32x4* src = reinterpret_cast<const f32x4*>(sk.partials) + slot * (BM * BN / 4) + in_slot;
            // a row of blocks at a time: all its loads are in flight together
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                f32x4 v[NI * 4];
#pragma unroll
                for (int q = 0; q < NI * 4; ++q) v[q] = __builtin_nontemporal_load(src + (i * NI * 4 + q) * 64);
                AXONN_FENCE();
#pragma unroll
                for (int q = 0; q < NI * 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[i][q / 4][4 * (q % 4) + e] += v[q][e];
                AXONN_FENCE();
            }
            // the slot is consumed: take its flag down again (a launch replayed from a captured HIP
            // graph carries the epoch of its capture)
            __syncthreads();
            if (t == 0) __hip_atomic_store(&sk.flags[slot], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- epilogue: fp32 -> bf16, transpose through this wave's private LDS region --------------
    // acc[i][j][4g + e] = C[m = i*32 + l%32][n = j*32 + 8g + 4*(l/32) + e]
    constexpr int CPR = TN / 8;   // 16-byte chunks per row of the wave tile (8 or 16)
    constexpr uint32_t CMASK = CPR - 1;
    const uint32_t half = lane >> 5, r32 = lane & 31;
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
                if (g == 3) AXONN_FENCE();   // convert block by block: keeps register pressure low
            }
    __syncthreads();
    uint16_t* pc = C + (m0 + wm * TM) * (int64_t)ldc + n0 + wn * TN;
    flush_c_block<TM, TN>(epi, pc, ldc, lane);
#undef AXONN_FENCE
}

}  // namespace axonn
