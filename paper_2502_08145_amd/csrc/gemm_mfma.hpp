// Building blocks shared by the bf16 x bf16 -> fp32 -> bf16 GEMM tile kernels for gfx950 (CDNA4):
//
//   C[M,N] = sum_k a(i,k) b(k,j)      (the local matrix multiply of Algorithm 1 lines 3, 11, 13)
//
//  * Global memory goes STRAIGHT into LDS (global_load_lds_dwordx4: 16 bytes per lane, no VGPR
//    staging, no LDS store instruction).
//  * An operand is either "K-contiguous" in global memory (A of NN/NT, B of NT) or
//    "MN-contiguous" (A of TN, B of NN/TN):
//      - K-contiguous panels of a 32-k stage sit in LDS as rows of 32 k (64 bytes) with the four
//        16-byte chunks of a row XOR-swizzled by the row number, and are read with ds_read_b128.
//        Their loads go out in pairs (two K-steps of the same rows back to back) so that both halves
//        of every 128-byte cache line are fetched together.
//      - MN-contiguous panels sit in LDS exactly as in memory, one LDS row per k, with the 16-byte
//        chunks of a k-row XOR-swizzled by k, and are read with the transposing ds_read_b64_tr_b16
//        (two per fragment).  No register transposes anywhere.
//    Because a direct load writes 1 KB of consecutive LDS per wave the swizzle is applied by
//    choosing WHICH 16 bytes of global memory each lane fetches.
//  * Loads and LDS reads are inline asm (the compiler would otherwise re-derive addresses with VALU
//    instructions and pick the 64-bit-VGPR addressing form); the waits on them are therefore written
//    out by hand too.
//  * Split-K state and the workgroup -> tile mapping: workgroup ids are remapped so that each of the
//    8 XCDs (which receive consecutive ids round-robin and have private L2s) works on a compact
//    patch of output tiles.
// The kernels themselves are gemm_tile_kernel16 (gemm_mfma16.hpp, 32-k LDS ring) and
// gemm_tile_kernel_k64 (gemm_mfma16_k64.hpp, 64-k stages).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace axonn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
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
//   cursor16(stage_off)        the VGPR addresses for reading that stage (made once per K-step)
//   read16<I>(frag, cursor)    fragment of 16-row block I: all 32 k of the stage
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
    const uint8_t* base[NBASE];                  // uniform: first row of load c (PAIR: of load 2c), k = 0
    uint32_t lds_dst[NBASE];                  // uniform: its destination inside stage 0
    uint32_t voff[2];                          // per lane: row-in-load * ld + fetched chunk * 16 + window
                                               // (+ 16 rows when the odd groups are served); [1]: one K-step on
    uint32_t lds_par;                          // uniform, PAIR: 1024 when the odd groups are served
    uint32_t step_add;                         // uniform, PAIR: what advance() adds to voff
    uint32_t raddr16;                          // read address of 16-row block 0 in stage 0

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
    using Frag = Frag128;
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
    const uint8_t* base;       // uniform: k-row 0 of the wave's first load; the K window moves here
    uint32_t voff[QL];         // per lane and load: k-row inside the wave's share * ld + fetched chunk * 16
    size_t kstep_bytes;        // uniform: KB k-rows
    uint32_t lds_dst[QL];
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
        const uint32_t sl = lane & 15, g = lane >> 4, kq = sl >> 2;
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
    using Frag = Frag64x2;
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
    int skew;             // 64-k kernels: every writer's K range is this much shorter than K / splits, the reader's longer by the sum
};
constexpr uint32_t kSplitSpinLimit = 1u << 19;   // x ~1 us per probe
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
            // any other count: range by range (writers first), and within a range the order of the
            // non-split case: the workgroups of the range that one XCD runs take consecutive tiles
            // (a tile's reader and writers then sit on different XCDs, which the exchange does not mind)
            w.krange = splits - 1 - pid / tiles;
            const int p = pid % tiles, j = p & 7, rem = tiles & 7;
            pid = j * (tiles >> 3) + (j < rem ? j : rem) + (p >> 3);
        }
        w.ktotal = K / splits;
    } else {
        // XCD x runs the workgroups x, x + 8, ...: nwg / 8 of them, one more on the first nwg % 8 XCDs; it
        // gets that many consecutive tiles of the sequence
        const int x = pid & 7, rem = nwg & 7;
        pid = x * (nwg >> 3) + (x < rem ? x : rem) + (pid >> 3);
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

}  // namespace axonn
