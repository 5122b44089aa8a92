// C ABI of the FC-layer GEMM library (see include/axonn_linear.h for the contract).
// Host side: argument checks, kernel-variant selection, launch.  No device memory is allocated
// anywhere in this file, and the GEMM entry points never synchronise: split-K kernels exchange their
// partial tiles through memory the caller registered (axonn_linear_set_workspace, which clears the
// flag words synchronously) or, for the one entry point made for callers that cannot allocate,
// through a file-scope device array.
#include "../../include/axonn_linear.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <map>
#include <mutex>
#include <tuple>

#include <vector>

#include "kernels.hpp"
#include "gemm_mfma16.hpp"       // tile configurations only: the kernels are instantiated in kernels_*.hip
#include "gemm_mfma16_k64.hpp"
#include "gemm_mfma16_k64p.hpp"
#include "gemm_edge.hpp"
#include "comm_model.hpp"
#include "transpose.hpp"

namespace axonn {

// ------------------------------------------------------------------------------------------
// Variant 0: guarded kernel, one thread per output element, any M, N, K >= 0.
// fp32 accumulation in ascending k, one RNE rounding at the store.
// ------------------------------------------------------------------------------------------
template <int LAYOUT>
__global__ __launch_bounds__(256) void gemm_naive_kernel(const uint16_t* __restrict__ A,
                                                         const uint16_t* __restrict__ B,
                                                         uint16_t* __restrict__ C, int64_t M,
                                                         int64_t N, int64_t K) {
    // 16 x 16 output blocks, numbered row-major, dealt out to the workgroups of a 1-D grid in turn
    const int64_t blocks_n = (N + 15) / 16, blocks = ((M + 15) / 16) * blocks_n;
    for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
        const int64_t j = (blk % blocks_n) * 16 + (threadIdx.x & 15);
        const int64_t i = (blk / blocks_n) * 16 + (threadIdx.x >> 4);
        if (i >= M || j >= N) continue;
        float acc = 0.f;
        for (int64_t k = 0; k < K; ++k) {
            const uint16_t a = (LAYOUT == AXONN_TN) ? A[k * M + i] : A[i * K + k];
            const uint16_t b = (LAYOUT == AXONN_NT) ? B[j * K + k] : B[k * N + j];
            acc += __builtin_bit_cast(float, (uint32_t)a << 16) * __builtin_bit_cast(float, (uint32_t)b << 16);
        }
        C[i * N + j] = (uint16_t)(pack2_bf16(acc, 0.f) & 0xFFFFu);
    }
}

// ------------------------------------------------------------------------------------------
// Variant table
// ------------------------------------------------------------------------------------------
struct Variant {
    const char* name;
    int bm, bn, threads, lds_bytes, min_k;  // bm == 0: the naive kernel; min_k per K range
    int kstep;                       // K (per range) must be a multiple of this
    int splits;                      // K ranges per tile (1: no split-K)
    bool k64;                        // the kernel with 64-k LDS stages
    // Throughput with every CU busy, per layout (NN, NT, TN), N(0,1) data, in units of about 1200 TFLOP/s.
    // `python -m paper_2502_08145_amd.sweeps variant_eff [--hot]` times every variant without split-K on
    // full-chip shapes and prints such a table.  The numbers below were taken that way as each kernel came
    // in; a re-measurement of all of them at once, with operands from HBM and with operands in cache,
    // gave tables whose plans ran the benchmark step and the model-zoo sweep 0.5-1 % slower (the small
    // tiles are picked for small outputs, which stay in cache, the large ones for large outputs, which
    // do not: neither condition alone describes both), so these stand.
    double eff[3];
    tile_kernel_t fn[3];             // per layout
    bool edge = false;               // the guarded MFMA kernel: any shape, launched through edge_kernel_launch
    int resident = 0;                // > 0: a grid of at most this many workgroups walks the tiles (one per compute unit)
};

// Kernel families: the 64-k-stage kernel (256 x 256, eight waves: the default wherever the output has
// whole large tiles), the 32-k ring (the same tile for NT at very long K and TN with four and more K
// ranges; the smaller tiles for outputs of few tiles), the guarded kernel.  Split-K variants of one
// tile share one kernel (the number of K ranges is a run-time argument).
static std::vector<Variant> make_variants() {
    std::vector<Variant> v;
    v.push_back({"naive", 0, 0, 256, 0, 0, 1, 1, false, {0, 0, 0}, {nullptr, nullptr, nullptr}});
    auto ring = [&](const char* name, int bm, int bn, int wn, int splits, int lds, int min_k, double nn, double nt, double tn) {
        Variant x{name, bm, bn, 128 * wn, lds, min_k, 2 * KB, splits, false, {nn, nt, tn}, {nullptr, nullptr, nullptr}};
        for (int l = 0; l < 3; ++l)
            x.fn[l] = (bm == 256 && bn == 256) ? ring_kernel_large(splits > 1, l) : ring_kernel_small(bm, bn, wn, splits > 1, l);
        v.push_back(x);
    };
    auto k64 = [&](const char* name, int splits) {
        Variant x{name, 256, 256, 512, k64_lds_bytes(256, 256, 1), TileCfgK64::MIN_K, TileCfgK64::KS, splits, true,
                  {1.17, 1.17, 1.15}, {nullptr, nullptr, nullptr}};
        for (int l = 0; l < 3; ++l) x.fn[l] = k64_kernel(splits > 1, l);
        v.push_back(x);
    };
    using L = TileCfg16<256, 256, 2, 4>;
    ring("mfma16_256x256_w8", 256, 256, 4, 1, L::LDS_BYTES, L::MIN_K, 1.13, 1.06, 1.12);
    static const char* const ring_sk[] = {"mfma16_256x256_w8_sk2", "mfma16_256x256_w8_sk3", "mfma16_256x256_w8_sk4", "mfma16_256x256_w8_sk5",
                                          "mfma16_256x256_w8_sk6", "mfma16_256x256_w8_sk7", "mfma16_256x256_w8_sk8"};
    for (int sp = 2; sp <= 8; ++sp) ring(ring_sk[sp - 2], 256, 256, 4, sp, L::LDS_BYTES, L::MIN_K, 1.13, 1.06, 1.12);
    ring("mfma16_256x128", 256, 128, 2, 1, TileCfg16<256, 128, 2, 2>::LDS_BYTES, TileCfg16<256, 128, 2, 2>::MIN_K, 0.86, 0.78, 0.91);
    ring("mfma16_128x256", 128, 256, 2, 1, TileCfg16<128, 256, 2, 2>::LDS_BYTES, TileCfg16<128, 256, 2, 2>::MIN_K, 0.95, 0.74, 0.92);
    ring("mfma16_128x256_w8", 128, 256, 4, 1, TileCfg16<128, 256, 2, 4>::LDS_BYTES, TileCfg16<128, 256, 2, 4>::MIN_K, 0.93, 0.72, 0.97);
    using S = TileCfg16<128, 128, 2, 2>;
    ring("mfma16_128x128", 128, 128, 2, 1, S::LDS_BYTES, S::MIN_K, 0.85, 0.72, 0.90);
    ring("mfma16_128x128_sk2", 128, 128, 2, 2, S::LDS_BYTES, S::MIN_K, 0.85, 0.72, 0.90);
    ring("mfma16_128x128_sk4", 128, 128, 2, 4, S::LDS_BYTES, S::MIN_K, 0.85, 0.72, 0.90);
    k64("mfma16k64_256x256_w8", 1);
    {
        Variant x{"mfma16k64p_256x256_w8", 256, 256, 512, TileCfgK64P::LDS_BYTES, TileCfgK64::MIN_K, TileCfgK64::KS, 1, true,
                  {1.20, 1.13, 1.17}, {nullptr, nullptr, nullptr}};
        for (int l = 0; l < 3; ++l) x.fn[l] = k64p_kernel(l);
        x.resident = TileCfgK64P::MAX_WORKGROUPS;
        v.push_back(x);
    }
    // half tiles with 64-k stages: NT only (eff from 2048 x 4096 x 4096 and 4096^3 against the ring's half tiles)
    auto k64h = [&](const char* name, int bm, int bn, int splits, double nt) {
        Variant x{name, bm, bn, 256, k64_lds_bytes(bm, bn, 3), TileCfgK64::MIN_K, TileCfgK64::KS, splits, true,
                  {0.0, nt, 0.0}, {nullptr, nullptr, nullptr}};
        for (int l = 0; l < 3; ++l) x.fn[l] = k64_kernel_half(bm, bn, splits > 1, l);
        v.push_back(x);
    };
    k64h("mfma16k64_256x128", 256, 128, 1, 0.95);
    k64h("mfma16k64_128x256", 128, 256, 1, 0.94);
    // split-K on the half tiles, for outputs that are narrow in one direction (2048 x 1152, 640 x 15360 ...) over a
    // long K: the 64-k kernel for NT, the 32-k ring for NN and TN
    // (two and three ranges only: with four and more the reader's turn at the slots costs more than the large
    // tile's split-K or 128 x 128 tiles do on the same outputs)
    static const char* const h1_sk[] = {"mfma16k64_256x128_sk2", "mfma16k64_256x128_sk3"};
    static const char* const h2_sk[] = {"mfma16k64_128x256_sk2", "mfma16k64_128x256_sk3"};
    static const char* const r1_sk[] = {"mfma16_256x128_sk2", "mfma16_256x128_sk3"};
    static const char* const r2_sk[] = {"mfma16_128x256_sk2", "mfma16_128x256_sk3"};
    for (int sp = 2; sp <= 3; ++sp) {
        k64h(h1_sk[sp - 2], 256, 128, sp, 0.85);
        k64h(h2_sk[sp - 2], 128, 256, sp, 0.84);
        ring(r1_sk[sp - 2], 256, 128, 2, sp, TileCfg16<256, 128, 2, 2>::LDS_BYTES, TileCfg16<256, 128, 2, 2>::MIN_K, 0.80, 0.70, 0.84);
        ring(r2_sk[sp - 2], 128, 256, 2, sp, TileCfg16<128, 256, 2, 2>::LDS_BYTES, TileCfg16<128, 256, 2, 2>::MIN_K, 0.80, 0.68, 0.82);
    }
    static const char* const k64_sk[] = {"mfma16k64_256x256_w8_sk2", "mfma16k64_256x256_w8_sk3", "mfma16k64_256x256_w8_sk4", "mfma16k64_256x256_w8_sk5",
                                         "mfma16k64_256x256_w8_sk6", "mfma16k64_256x256_w8_sk7", "mfma16k64_256x256_w8_sk8"};
    for (int sp = 2; sp <= 8; ++sp) k64(k64_sk[sp - 2], sp);
    // guarded MFMA kernel: ragged shapes and the edge strips of ragged outputs
    Variant e{"mfma16_edge_128x128", EdgeCfg::BM, EdgeCfg::BN, EdgeCfg::NT, EdgeCfg::LDS_BYTES, 1, 1, 1, false, {0, 0, 0}, {nullptr, nullptr, nullptr}};
    e.edge = true;
    v.push_back(e);
    return v;
}
static const std::vector<Variant>& variants() {
    static const std::vector<Variant> table = make_variants();
    return table;
}
static int num_variants() { return (int)variants().size(); }
static int edge_variant() { return num_variants() - 1; }
static bool is_guarded(int v) { return variants()[v].bm == 0 || variants()[v].edge; }

// Split-K scratch: one area per device.  Layout: kFlagBytes of flags (one 32-bit flag per slot, the
// time-out counter in the last word), then slots of one 256x256 fp32 tile each.  The area is the
// caller's (axonn_linear_set_workspace); without one the three GEMM entry points run the kernels that
// need none.  The library itself allocates nothing.
constexpr int kScratchSlots = 256;                          // the most any variant is allowed to need
constexpr size_t kSlotBytes = 256 * 256 * sizeof(float);
constexpr size_t kFlagBytes = 4096;                         // 1023 flags + the counter
constexpr int64_t kMaxFlags = kFlagBytes / sizeof(uint32_t) - 1;
constexpr int kMaxDevices = 64;
struct Scratch {
    float* partials = nullptr;
    uint32_t* flags = nullptr;
    size_t partial_bytes = 0;       // capacity behind `partials`
    uint32_t* timeouts() const { return flags + kFlagBytes / sizeof(uint32_t) - 1; }
};
static Scratch g_scratch[kMaxDevices];
static std::mutex g_scratch_mutex;
static std::atomic<uint32_t> g_epoch{0};
static std::atomic<int> g_split_k_enabled{1};

static Scratch carve(void* p, size_t bytes) {
    Scratch sc;
    sc.flags = static_cast<uint32_t*>(p);
    sc.partials = reinterpret_cast<float*>(static_cast<char*>(p) + kFlagBytes);
    sc.partial_bytes = bytes - kFlagBytes;
    return sc;
}

// The current device's registered area (by value: a later set_workspace does not disturb a launch
// being prepared) if it has room for `bytes_needed` bytes of partial tiles; else .partials == nullptr.
static Scratch registered_scratch(size_t bytes_needed) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return Scratch{};
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    const Scratch& sc = g_scratch[dev];
    return (sc.partials && sc.partial_bytes >= bytes_needed) ? sc : Scratch{};
}

// The scratch area of the entry point for callers that cannot allocate: a device array of fixed size
// that every GPU the library runs on holds from the moment the code object is loaded until the
// process ends (zero-filled at load).  In host code the array's NAME is only a handle for
// hipGetSymbolAddress; the address kernels and copies may use is looked up once per device, with that
// device current, and kept in g_static_ptr.
constexpr int kStaticSlots = 128;                           // 32 MiB of partial tiles
constexpr size_t kStaticBytes = kFlagBytes + kStaticSlots * kSlotBytes;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticBytes];
static unsigned char* g_static_ptr[kMaxDevices];
static std::mutex g_static_mutex;

// The current device's copy of the static area; .partials == nullptr if the look-up failed.
static Scratch static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return Scratch{};
    }
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return Scratch{};
        }
        g_static_ptr[dev] = static_cast<unsigned char*>(p);
    }
    return carve(g_static_ptr[dev], kStaticBytes);
}

static std::atomic<int> g_forced{-1};
static std::once_flag g_attr_once[kMaxDevices];   // the LDS limits are a per-device property of a kernel

static bool variant_supports(int v, int64_t M, int64_t N, int64_t K, int layout) {
    if (v < 0 || v >= num_variants() || layout < 0 || layout > 2) return false;
    const Variant& var = variants()[v];
    if (var.bm == 0) return true;
    if (M <= 0 || N <= 0 || K <= 0) return false;
    if (var.edge) return ((M + var.bm - 1) / var.bm) * ((N + var.bn - 1) / var.bn) < ((int64_t)1 << 31);
    if (!var.fn[layout]) return false;   // a kernel for one layout only
    // per-lane address offsets are 32 bits: up to 16 rows of a K-contiguous operand, 4 (64-k kernel: 36)
    // k-rows of an MN-contiguous one, plus the K window of a K-contiguous one
    constexpr int64_t kMaxTileDim = (int64_t)1 << 24;
    if (M > kMaxTileDim || N > kMaxTileDim || K > kMaxTileDim) return false;
    if (M % var.bm != 0 || N % var.bn != 0 || K % (var.kstep * var.splits) != 0 || K / var.splits < var.min_k) return false;
    if (var.splits == 1) return true;
    // scratch: one flag and one fp32 tile per (tile, extra K range)
    const int64_t slots = (M / var.bm) * (N / var.bn) * (var.splits - 1);
    return slots <= kMaxFlags && slots * var.bm * var.bn * (int64_t)sizeof(float) <= (int64_t)(kScratchSlots * kSlotBytes);
}

// Tile-shape choice.  MI355X has 256 compute units; a partly filled last round of tiles costs a
// whole tile time, and a smaller tile moves more operand bytes per flop.  Pick the variant with the
// smallest modelled time:
//     rounds x tile area x (K per workgroup + fixed cost) / efficiency
// where the efficiencies are throughputs measured on MI355X with every CU busy (N(0,1) data, see
// Variant::eff), and the fixed cost (pipeline fill, epilogue,
// for split-K also the exchange of fp32 partial tiles) is expressed in units of k.
// K-contiguous operands are the dearer ones to stage (64-byte row segments per load), which is
// why NN likes a short A tile (128x256) and NT gains least from any of the smaller tiles.
// Split-K turns an output of at most 128 tiles of 256x256 into a full round of the large tile.
static double model_time(int v, int64_t M, int64_t N, int64_t K, int layout, bool allow_split) {
    constexpr double kFixedK = 128.0;
    const Variant& var = variants()[v];
    if (!variant_supports(v, M, N, K, layout) || (var.splits > 1 && !allow_split) || var.eff[layout] <= 0.0) return -1.0;
    // Long K: without split-K the 64-k kernels lead the 32-k ring in every mode (8192 x 8192 x 32768 and
    // x 49152: NN and TN by 1-5 %, NT, since its A panel is triple-buffered, by 9-10 %).  With split-K
    // they lead in NN and NT at any K tried (2048 x 2048 x 65536 in four ranges: +5 % and +11 %;
    // 1024 x 2048 x 131072 in eight: +3 % and +13 %), in TN the ring is level or up to 8 % ahead above
    // K = 32768.
    if (var.k64 && var.splits > 1 && layout == AXONN_TN && K > 32768) return -1.0;
    // The resident-workgroup form of the 64-k kernel: measured against one workgroup per tile in the
    // benchmark's sequence, 1.3-1.9 % less time for the TN products of three and four tiles per compute
    // unit, +-1 % for NN, 1.6 % MORE for NT with two tiles and 2.5 % more with a single tile.
    // What it saves is per tile: at K = 16384 and 32768 it measures 2.5-5 % behind one workgroup per tile.
    // NN at K = 2048 (4096 x 16384 x 2048, four tiles per compute unit): 226 -> 220 us.
    if (var.resident > 0 && !((layout == AXONN_TN || (layout == AXONN_NN && K <= 2048)) && (M / var.bm) * (N / var.bn) >= 3 * var.resident && K <= 8192)) return -1.0;
    const int64_t wgs = (M / var.bm) * (N / var.bn) * var.splits;
    // Every CU works through ceil(wgs / 256) workgroups (two small tiles resident on one CU run
    // side by side at half speed each, which comes to the same).  A last round that fills only
    // a fraction f of the CUs runs faster than a full one (the busy CUs get the idle ones'
    // power and bandwidth): measured about 0.6 + 0.4 f of a full round (0.61 at 4 workgroups,
    // 0.78 at 128, 0.87 at 144).
    const int64_t full = wgs / 256, rest = wgs % 256;
    // readers and writers of a tile should run side by side: one round of large tiles, two of small ones
    if (var.splits > 1 && wgs > (var.bm * var.bn <= 128 * 128 ? 512 : 256)) return -1.0;
    const double rounds = (double)full + (rest ? 0.6 + 0.4 * (double)rest / 256.0 : 0.0);
    // the exchange of a small tile is latency: the reader takes the partial tiles one after the
    // other once the writers are done, and it grows with the number of tiles in flight
    // (measured: 4 us + 0.055 us per tile for two K ranges, 7 us + 0.17 us per tile for four)
    const double tiles = (double)((M / var.bm) * (N / var.bn));
    const double fixed_small = var.splits == 2 ? 700.0 + 8.0 * tiles : 1300.0 + 25.0 * tiles;
    // large tiles: the partial tiles travel through HBM, (splits - 1) x 256 KB per tile written and
    // read back at 4-5 TB/s (0.1 us, or 4 units of k, per slot), and the reader of a tile takes its
    // slots one after the other at one CU's rate (2.5 us, 100 units, per slot)
    // (half tiles: half the bytes per slot in flight; what the reader pays per slot is mostly latency)
    const bool half_tile = var.bm * var.bn < 256 * 256;
    const double fixed_large = 4.0 * tiles * (var.splits - 1) * (var.bm * var.bn) / 65536.0 + (half_tile ? 160.0 : 100.0) * (var.splits - 1);
    const double k_cost = (double)(K / var.splits) + kFixedK +
                          (var.splits == 1 ? 0.0 : var.bm * var.bn <= 128 * 128 ? fixed_small : fixed_large);
    double e = var.eff[layout];
    // the 64-k kernel leads the 32-k ring in TN by 2-4 % in one range and in two (six clusters of
    // transposing reads, streamed epilogue); with four ranges and more it measured 2-4 % behind
    if (layout == AXONN_TN && var.k64 && var.splits >= 4) e *= 0.94;
    return rounds * var.bm * var.bn * k_cost / e;
}

// What the guarded MFMA kernel takes for an m x n block, in the model's units (2.6e6 to the
// microsecond: a 256 x 256 tile over K = 4096 is 2.7e8 and takes about 100 us).  Its K-steps of
// 128 are a chain of load, barrier, LDS store, barrier, multiply: measured 1.9 us per step for a
// workgroup that has a compute unit to itself, 1.6 us with the chip full (two to a CU, 205 us for
// 4096^3 in 1024 workgroups), plus launch and epilogue.
static double edge_time(int64_t m, int64_t n, int64_t K) {
    const double wgs = (double)(((m + EdgeCfg::BM - 1) / EdgeCfg::BM) * ((n + EdgeCfg::BN - 1) / EdgeCfg::BN));
    const double steps = (double)((K + EdgeCfg::BK - 1) / EdgeCfg::BK);
    return (3.0 + steps * 2.0 * std::max(1.0, wgs / 320.0)) * 2.6e6;
}

// The variant with the smallest modelled time for one launch over the whole output (the guarded MFMA
// kernel if no tile shape divides it; 0, the naive kernel, for K = 0); *t_out receives that time.
static int select_variant(int64_t M, int64_t N, int64_t K, int layout, bool allow_split, double* t_out = nullptr) {
    int best = 0;
    double best_t = 0;
    for (int v = 1; v < num_variants(); ++v) {
        const double t = model_time(v, M, N, K, layout, allow_split);
        if (t >= 0.0 && (best == 0 || t < best_t)) {
            best = v;
            best_t = t;
        }
    }
    if (best == 0 && variant_supports(edge_variant(), M, N, K, layout)) {
        best = edge_variant();
        best_t = edge_time(M, N, K);
    }
    if (t_out) *t_out = best_t;
    return best;
}

// A product as one launch, or as two launches over disjoint blocks of the output.  An output of,
// say, 384 large tiles keeps the 256 CUs busy for one round and half of them for a second; cut
// into a block of 256 tiles and a block of 128, the second block can run as split-K (or on a
// smaller tile) and fill the chip again.  The cut runs along N (the second block holds the last
// columns) or along M (the last rows); operand and output blocks are addressed through the leading
// dimensions of the whole matrices.
struct Part {
    int variant;
    int64_t m, n, row0, col0;
};
struct Plan {
    int parts;
    Part part[AXONN_MAX_PLAN_PARTS];
};
static_assert(AXONN_MAX_PLAN_PARTS >= 4, "two launches over whole tiles and two edge strips");

static Plan make_plan(int64_t M, int64_t N, int64_t K, int layout, bool allow_split) {
    double t_one = 0;
    Plan plan{1, {{select_variant(M, N, K, layout, allow_split, &t_one), M, N, 0, 0}}};
    if (is_guarded(plan.part[0].variant)) {
        // Ragged output of some size: the whole 128 x 128 tiles go to the tile kernels (if K suits
        // them), the last columns and the last rows to the guarded kernel, as strips of their own.
        const int64_t mm = M - M % 128, nm = N - N % 128;
        // the tile kernels move 16 bytes at a time: every row of the operands and of the output, as
        // stored in the whole matrices, has to start on a 16-byte boundary (K is a multiple of 32 here)
        const bool rows_aligned = N % 8 == 0 && (layout != AXONN_TN || M % 8 == 0);
        if (mm > 0 && nm > 0 && (mm != M || nm != N) && rows_aligned) {
            constexpr double kNextLaunch = 8.0e6;   // about 3 us, as for the two-launch plans below
            double t_tiles = 0;
            const int v_tiles = select_variant(mm, nm, K, layout, allow_split, &t_tiles);
            const double t_strips = (nm != N ? edge_time(mm, N - nm, K) + kNextLaunch : 0.0) +
                                    (mm != M ? edge_time(M - mm, N, K) + kNextLaunch : 0.0);
            if (!is_guarded(v_tiles) && t_tiles + t_strips < t_one) {
                const Plan inner = make_plan(mm, nm, K, layout, allow_split);
                plan = inner;
                if (nm != N) plan.part[plan.parts++] = Part{edge_variant(), mm, N - nm, 0, nm};
                if (mm != M) plan.part[plan.parts++] = Part{edge_variant(), M - mm, N, mm, 0};
            }
        }
        return plan;
    }
    // nothing to gain within half a round of large tiles: split-K and the smaller tiles cover that
    if (M % 128 != 0 || N % 128 != 0 || (M / 128) * (N / 128) <= 4 * 128) return plan;
    // what a second launch costs beyond its own fill and drain (the first one's tail is not
    // overlapped), in the model's units: about 3 us
    constexpr double kSecondLaunch = 8.0e6;
    // a two-launch plan must be clearly better: the model is good to a few per cent
    double best_t = t_one * 0.97;
    auto consider = [&](bool along_n, int64_t rest) {
        const int64_t m1 = along_n ? M : M - rest, n1 = along_n ? N - rest : N;
        const int64_t m2 = along_n ? M : rest, n2 = along_n ? rest : N;
        double t1 = 0, t2 = 0;
        const int v1 = select_variant(m1, n1, K, layout, allow_split, &t1);
        const int v2 = select_variant(m2, n2, K, layout, allow_split, &t2);
        if (is_guarded(v1) || is_guarded(v2) || t1 + t2 + kSecondLaunch >= best_t) return;
        best_t = t1 + t2 + kSecondLaunch;
        plan = Plan{2, {{v1, m1, n1, 0, 0}, {v2, m2, n2, along_n ? 0 : m1, along_n ? n1 : 0}}};
    };
    // second blocks of up to half a round of large tiles, in steps of one tile column / row
    const int64_t step_n = N % 256 == 0 ? 256 : 128, step_m = M % 256 == 0 ? 256 : 128;
    for (int64_t rest = step_n; rest < N && M * rest <= (int64_t)128 * 256 * 256; rest += step_n) consider(true, rest);
    for (int64_t rest = step_m; rest < M && rest * N <= (int64_t)128 * 256 * 256; rest += step_m) consider(false, rest);
    return plan;
}

// Plans are remembered per shape: the search above costs a few hundred model evaluations.
static std::map<std::tuple<int64_t, int64_t, int64_t, int, bool>, Plan> g_plans;
static std::mutex g_plans_mutex;

static Plan cached_plan(int64_t M, int64_t N, int64_t K, int layout, bool allow_split) {
    const auto key = std::make_tuple(M, N, K, layout, allow_split);
    {
        std::lock_guard<std::mutex> lock(g_plans_mutex);
        const auto it = g_plans.find(key);
        if (it != g_plans.end()) return it->second;
    }
    const Plan plan = make_plan(M, N, K, layout, allow_split);
    std::lock_guard<std::mutex> lock(g_plans_mutex);
    if (g_plans.size() >= 4096) g_plans.clear();
    g_plans[key] = plan;
    return plan;
}

static int check_args(int64_t M, int64_t N, int64_t K, int layout, const void* a, const void* b,
                      void* c, int fp32_accumulate) {
    constexpr int64_t kMaxDim = (int64_t)1 << 31, kMaxElems = (int64_t)1 << 40;
    if (M < 0 || N < 0 || K < 0 || M >= kMaxDim || N >= kMaxDim || K >= kMaxDim) return AXONN_ERR_INVALID_ARG;
    if (layout < 0 || layout > 2) return AXONN_ERR_INVALID_ARG;
    if (fp32_accumulate != 0 && fp32_accumulate != 1) return AXONN_ERR_INVALID_ARG;
    if (M * K >= kMaxElems || K * N >= kMaxElems || M * N >= kMaxElems) return AXONN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return AXONN_OK;
    if (!c || (reinterpret_cast<uintptr_t>(c) & 15)) return AXONN_ERR_INVALID_ARG;
    if (K > 0) {
        if (!a || !b) return AXONN_ERR_INVALID_ARG;
        if ((reinterpret_cast<uintptr_t>(a) & 15) || (reinterpret_cast<uintptr_t>(b) & 15))
            return AXONN_ERR_INVALID_ARG;
    }
    return AXONN_OK;
}

static void raise_lds_limits() {
    for (const Variant& var : variants())
        for (int l = 0; l < 3; ++l)
            if (var.fn[l])
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(var.fn[l]), hipFuncAttributeMaxDynamicSharedMemorySize, var.lds_bytes);
    edge_kernel_raise_lds_limit();
    (void)hipGetLastError();
}

// once per device, the first time a kernel that needs it is about to be launched there
static void raise_lds_limits_once() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        raise_lds_limits();
        return;
    }
    std::call_once(g_attr_once[dev], raise_lds_limits);
}

static size_t split_bytes(const Part& p) {
    const Variant& x = variants()[p.variant];
    return x.splits == 1 ? 0 : (size_t)((p.m / x.bm) * (p.n / x.bn) * (x.splits - 1)) * x.bm * x.bn * sizeof(float);
}

static size_t split_bytes(const Plan& plan) {
    size_t bytes = 0;
    for (int i = 0; i < plan.parts; ++i) bytes = std::max(bytes, split_bytes(plan.part[i]));
    return bytes;   // the launches of a plan run one after the other and share the area
}

// workgroups of the launch over block `p`
static int64_t part_workgroups(const Part& p) {
    const Variant& var = variants()[p.variant];
    return ((p.m + var.bm - 1) / var.bm) * ((p.n + var.bn - 1) / var.bn) * var.splits;
}

// One kernel launch over the block `p` of the M x N output.
static void launch_part(const Part& p, int64_t M, int64_t N, int64_t K, int layout, const uint16_t* A, const uint16_t* B,
                        uint16_t* C, const Scratch& scratch, hipStream_t s) {
    const Variant& var = variants()[p.variant];
    const int64_t lda = layout == AXONN_TN ? M : K, ldb = layout == AXONN_NT ? K : N, ldc = N;
    A += layout == AXONN_TN ? p.row0 : p.row0 * K;
    B += layout == AXONN_NT ? p.col0 * K : p.col0;
    C += p.row0 * N + p.col0;
    if (var.edge) {
        const int tiles_n = (int)((p.n + var.bn - 1) / var.bn);
        edge_kernel_launch(layout, (unsigned)part_workgroups(p), s, A, B, C, p.m, p.n, K, lda, ldb, ldc, tiles_n);
        return;
    }
    const int tiles_m = (int)(p.m / var.bm), tiles_n = (int)(p.n / var.bn);
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int group_m = tiles_m < 8 ? tiles_m : 8;
    SplitK sk{nullptr, nullptr, nullptr, 0u, 1, 0};
    if (var.splits > 1) {
        uint32_t epoch = g_epoch.fetch_add(1, std::memory_order_relaxed) + 1;
        if (epoch == 0) epoch = g_epoch.fetch_add(1, std::memory_order_relaxed) + 1;   // flags start at 0
        // one iteration less for every writer (measured on 2048 x 4096 x 4096 and x 16384 in two ranges: 64 k
        // takes 1-2 us off, 128 and more give it back)
        const int skew = (var.k64 && K / var.splits >= 1024) ? TileCfgK64::KS : 0;
        sk = SplitK{scratch.partials, scratch.flags, scratch.timeouts(), epoch, var.splits, skew};
    }
    const int64_t grid = var.resident > 0 ? std::min<int64_t>(tiles, var.resident) : tiles * var.splits;
    hipLaunchKernelGGL(var.fn[layout], dim3((unsigned)grid), dim3(var.threads), var.lds_bytes, s,
                       A, B, C, (int)K, (int)lda, (int)ldb, (int)ldc, tiles_m, tiles_n, group_m, sk);
}

// Where a call's split-K kernels find their scratch area.
enum class ScratchFrom { Registered, Static };

static int launch(int64_t M, int64_t N, int64_t K, int layout, const void* a, const void* b, void* c,
                  int fp32_accumulate, void* stream, ScratchFrom from = ScratchFrom::Registered) {
    const int rc = check_args(M, N, K, layout, a, b, c, fp32_accumulate);
    if (rc != AXONN_OK) return rc;
    if (M == 0 || N == 0) return AXONN_OK;

    const int forced = g_forced.load(std::memory_order_relaxed);
    Plan plan;
    Scratch scratch;
    if (forced >= 0) {
        if (!variant_supports(forced, M, N, K, layout)) return AXONN_ERR_UNSUPPORTED;
        plan = Plan{1, {{forced, M, N, 0, 0}}};
    } else {
        plan = cached_plan(M, N, K, layout, g_split_k_enabled.load(std::memory_order_relaxed) != 0);
    }
    if (const size_t need = split_bytes(plan)) {
        if (from == ScratchFrom::Static) {
            // the static area has one size: a product whose plan needs more is refused, not re-planned
            if (need > kStaticSlots * kSlotBytes || !(scratch = static_scratch()).partials) return AXONN_ERR_WORKSPACE;
        } else if (!(scratch = registered_scratch(need)).partials) {
            if (forced >= 0) return AXONN_ERR_WORKSPACE;
            plan = cached_plan(M, N, K, layout, false);   // no area, or too small a one: the kernels that need none
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t* A = static_cast<const uint16_t*>(a);
    const uint16_t* B = static_cast<const uint16_t*>(b);
    uint16_t* C = static_cast<uint16_t*>(c);

    (void)hipGetLastError();
    if (variants()[plan.part[0].variant].bm == 0) {
        const int64_t blocks = ((M + 15) / 16) * ((N + 15) / 16);
        const dim3 grid((unsigned)std::min<int64_t>(blocks, (int64_t)1 << 20));
        switch (layout) {
            case AXONN_NN: hipLaunchKernelGGL(gemm_naive_kernel<AXONN_NN>, grid, dim3(256), 0, s, A, B, C, M, N, K); break;
            case AXONN_NT: hipLaunchKernelGGL(gemm_naive_kernel<AXONN_NT>, grid, dim3(256), 0, s, A, B, C, M, N, K); break;
            default:       hipLaunchKernelGGL(gemm_naive_kernel<AXONN_TN>, grid, dim3(256), 0, s, A, B, C, M, N, K); break;
        }
    } else {
        raise_lds_limits_once();
        for (int i = 0; i < plan.parts; ++i)
            if (part_workgroups(plan.part[i]) >= ((int64_t)1 << 31)) return AXONN_ERR_UNSUPPORTED;
        for (int i = 0; i < plan.parts; ++i) launch_part(plan.part[i], M, N, K, layout, A, B, C, scratch, s);
    }
    return hipGetLastError() == hipSuccess ? AXONN_OK : AXONN_ERR_LAUNCH;
}

// ------------------------------------------------------------------------------------------
// Mode tuner (paper Sec. IV-C): time a product in all three modes once, remember the result.
// ------------------------------------------------------------------------------------------
static std::map<std::tuple<int, int64_t, int64_t, int64_t>, axonn_tune_result_t> g_tuned;
static std::mutex g_tuned_mutex;

static bool first_is_mk(int mode) { return mode != AXONN_TN; }
static bool second_is_kn(int mode) { return mode != AXONN_NT; }

// Mean time in microseconds of `reps` runs of f() on stream s (after `warm` untimed ones); < 0 on error.
template <class F>
static float time_us(hipStream_t s, int warm, int reps, F&& f) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return -1.f;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return -1.f;
    }
    bool ok = true;
    for (int i = 0; i < warm && ok; ++i) ok = f() == AXONN_OK;
    ok = ok && hipEventRecord(e0, s) == hipSuccess;
    for (int i = 0; i < reps && ok; ++i) ok = f() == AXONN_OK;
    ok = ok && hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
    float ms = 0.f;
    ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ok ? ms * 1000.f / (float)reps : -1.f;
}

}  // namespace axonn

extern "C" {

int axonn_linear_tune(int op, int64_t M, int64_t N, int64_t K, const void* first, const void* second, void* out,
                      void* scratch, size_t scratch_bytes, void* stream, axonn_tune_result_t* result) {
    using namespace axonn;
    if (op < 0 || op > 2 || !result || M <= 0 || N <= 0 || K <= 0) return AXONN_ERR_INVALID_ARG;
    const int nat = op;   // fwd: NN, bwd_data: NT, bwd_weight: TN -- the modes the cached buffers give for free
    int rc = check_args(M, N, K, nat, first, second, out, 1);
    if (rc != AXONN_OK) return rc;
    if (scratch_bytes && (!scratch || (reinterpret_cast<uintptr_t>(scratch) & 255))) return AXONN_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t first_bytes = (((size_t)M * K * 2) + 255) & ~(size_t)255, second_bytes = (size_t)K * N * 2;
    axonn_tune_result_t r;
    r.best_layout = r.best_layout_all_in = nat;
    float best = -1.f, best_all = -1.f;
    for (int m = 0; m < 3; ++m) {
        r.gemm_us[m] = -1.f;
        r.restore_first_us[m] = r.restore_second_us[m] = 0.f;
        const bool tf = first_is_mk(m) != first_is_mk(nat), ts = second_is_kn(m) != second_is_kn(nat);
        const size_t need = (tf ? first_bytes : 0) + (ts ? second_bytes : 0);
        if (need > scratch_bytes) continue;   // this mode cannot be tried
        const void* a = first;
        const void* b = second;
        char* free_ptr = static_cast<char*>(scratch);
        if (tf) {
            const int64_t rows = first_is_mk(nat) ? M : K, cols = first_is_mk(nat) ? K : M;
            void* dst = free_ptr;
            free_ptr += first_bytes;
            r.restore_first_us[m] = time_us(s, 1, 3, [&] { return axonn_transpose_bf16(rows, cols, first, dst, stream); });
            if (r.restore_first_us[m] < 0.f) return AXONN_ERR_LAUNCH;
            a = dst;
        }
        if (ts) {
            const int64_t rows = second_is_kn(nat) ? K : N, cols = second_is_kn(nat) ? N : K;
            void* dst = free_ptr;
            r.restore_second_us[m] = time_us(s, 1, 3, [&] { return axonn_transpose_bf16(rows, cols, second, dst, stream); });
            if (r.restore_second_us[m] < 0.f) return AXONN_ERR_LAUNCH;
            b = dst;
        }
        r.gemm_us[m] = time_us(s, 2, 5, [&] { return launch(M, N, K, m, a, b, out, 1, stream); });
        if (r.gemm_us[m] < 0.f) return AXONN_ERR_LAUNCH;
        // the weight (second operand of fwd and bwd_data) changes once per optimiser step, the other
        // operands with every call: only their re-storage is charged to the call
        const float all_in = r.gemm_us[m] + r.restore_first_us[m] + (op == 2 ? r.restore_second_us[m] : 0.f);
        if (best < 0.f || r.gemm_us[m] < best) {
            best = r.gemm_us[m];
            r.best_layout = m;
        }
        if (best_all < 0.f || all_in < best_all) {
            best_all = all_in;
            r.best_layout_all_in = m;
        }
    }
    {
        std::lock_guard<std::mutex> lock(g_tuned_mutex);
        g_tuned[std::make_tuple(op, M, N, K)] = r;
    }
    *result = r;
    return AXONN_OK;
}

int axonn_linear_tuned(int op, int64_t M, int64_t N, int64_t K, axonn_tune_result_t* result) {
    if (op < 0 || op > 2 || !result) return AXONN_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(axonn::g_tuned_mutex);
    auto it = axonn::g_tuned.find(std::make_tuple(op, M, N, K));
    if (it == axonn::g_tuned.end()) return 0;
    *result = it->second;
    return 1;
}

int axonn_linear_tuned_set(int op, int64_t M, int64_t N, int64_t K, const axonn_tune_result_t* result) {
    if (op < 0 || op > 2 || !result || M <= 0 || N <= 0 || K <= 0 || result->best_layout < 0 || result->best_layout > 2 ||
        result->best_layout_all_in < 0 || result->best_layout_all_in > 2)
        return AXONN_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(axonn::g_tuned_mutex);
    axonn::g_tuned[std::make_tuple(op, M, N, K)] = *result;
    return AXONN_OK;
}

int axonn_linear_tuned_call(int op, int64_t M, int64_t N, int64_t K, const void* first, const void* second, void* out,
                            const void* second_restored, void* scratch, size_t scratch_bytes, int fp32_accumulate,
                            void* stream, int* layout_used) {
    using namespace axonn;
    if (op < 0 || op > 2) return AXONN_ERR_INVALID_ARG;
    const int nat = op;
    int rc = check_args(M, N, K, nat, first, second, out, fp32_accumulate);
    if (rc != AXONN_OK) return rc;
    if (scratch_bytes && (!scratch || (reinterpret_cast<uintptr_t>(scratch) & 255))) return AXONN_ERR_INVALID_ARG;
    if (second_restored && (reinterpret_cast<uintptr_t>(second_restored) & 15)) return AXONN_ERR_INVALID_ARG;
    int mode = nat;
    {
        std::lock_guard<std::mutex> lock(g_tuned_mutex);
        const auto it = g_tuned.find(std::make_tuple(op, M, N, K));
        if (it != g_tuned.end()) mode = it->second.best_layout_all_in;
    }
    bool tf = first_is_mk(mode) != first_is_mk(nat), ts = second_is_kn(mode) != second_is_kn(nat);
    const size_t first_bytes = (((size_t)M * K * 2) + 255) & ~(size_t)255, second_bytes = (size_t)K * N * 2;
    const size_t need = (tf ? first_bytes : 0) + ((ts && !second_restored) ? second_bytes : 0);
    if (need > scratch_bytes || M == 0 || N == 0 || K == 0) {   // no room to re-store: the natural mode needs none
        mode = nat;
        tf = ts = false;
    }
    const void* a = first;
    const void* b = second;
    char* free_ptr = static_cast<char*>(scratch);
    if (tf) {
        const int64_t rows = first_is_mk(nat) ? M : K, cols = first_is_mk(nat) ? K : M;
        rc = axonn_transpose_bf16(rows, cols, first, free_ptr, stream);
        if (rc != AXONN_OK) return rc;
        a = free_ptr;
        free_ptr += first_bytes;
    }
    if (ts) {
        if (second_restored) {
            b = second_restored;
        } else {
            const int64_t rows = second_is_kn(nat) ? K : N, cols = second_is_kn(nat) ? N : K;
            rc = axonn_transpose_bf16(rows, cols, second, free_ptr, stream);
            if (rc != AXONN_OK) return rc;
            b = free_ptr;
        }
    }
    if (layout_used) *layout_used = mode;
    return launch(M, N, K, mode, a, b, out, fp32_accumulate, stream);
}

void axonn_linear_tune_reset(void) {
    std::lock_guard<std::mutex> lock(axonn::g_tuned_mutex);
    axonn::g_tuned.clear();
}

int axonn_linear_fwd(int64_t M, int64_t N, int64_t K, int layout, const void* X, const void* W, void* Y,
                     int fp32_accumulate, void* stream) {
    return axonn::launch(M, N, K, layout, X, W, Y, fp32_accumulate, stream);
}

int axonn_linear_bwd_data(int64_t M, int64_t N, int64_t K, int layout, const void* dY, const void* W, void* dX,
                          int fp32_accumulate, void* stream) {
    return axonn::launch(M, N, K, layout, dY, W, dX, fp32_accumulate, stream);
}

int axonn_linear_bwd_weight(int64_t M, int64_t N, int64_t K, int layout, const void* X, const void* dY, void* dW,
                            int fp32_accumulate, void* stream) {
    return axonn::launch(M, N, K, layout, X, dY, dW, fp32_accumulate, stream);
}

int axonn_linear_gemm_static(int64_t M, int64_t N, int64_t K, int layout, const void* first, const void* second, void* out,
                             int fp32_accumulate, void* stream) {
    return axonn::launch(M, N, K, layout, first, second, out, fp32_accumulate, stream, axonn::ScratchFrom::Static);
}

size_t axonn_linear_static_scratch_bytes(void) { return axonn::kStaticBytes; }

const char* axonn_status_string(int status) {
    switch (status) {
        case AXONN_OK: return "ok";
        case AXONN_ERR_INVALID_ARG: return "invalid argument (null or misaligned pointer, bad dimension, layout or flag)";
        case AXONN_ERR_UNSUPPORTED: return "the forced kernel variant cannot run this shape";
        case AXONN_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        case AXONN_ERR_WORKSPACE: return "no split-K scratch area of the size needed (none registered, the registered one too small, or the product's plan exceeds the static area)";
        default: return "unknown status";
    }
}

int axonn_linear_version(void) { return 100; }

int axonn_linear_num_variants(void) { return axonn::num_variants(); }

const char* axonn_linear_variant_name(int variant) {
    return (variant >= 0 && variant < axonn::num_variants()) ? axonn::variants()[variant].name : nullptr;
}

int axonn_linear_variant_supports(int variant, int64_t M, int64_t N, int64_t K, int layout) {
    return axonn::variant_supports(variant, M, N, K, layout) ? 1 : 0;
}

int axonn_linear_select_variant(int64_t M, int64_t N, int64_t K, int layout) {
    if (M < 0 || N < 0 || K < 0 || layout < 0 || layout > 2) return AXONN_ERR_INVALID_ARG;
    return axonn::select_variant(M, N, K, layout, axonn::g_split_k_enabled.load(std::memory_order_relaxed) != 0);
}

int axonn_linear_plan(int64_t M, int64_t N, int64_t K, int layout, axonn_plan_part_t parts[AXONN_MAX_PLAN_PARTS]) {
    if (M <= 0 || N <= 0 || K < 0 || layout < 0 || layout > 2 || !parts) return AXONN_ERR_INVALID_ARG;
    const axonn::Plan plan = axonn::cached_plan(M, N, K, layout, axonn::g_split_k_enabled.load(std::memory_order_relaxed) != 0);
    for (int i = 0; i < plan.parts; ++i)
        parts[i] = axonn_plan_part_t{plan.part[i].variant, plan.part[i].m, plan.part[i].n, plan.part[i].row0, plan.part[i].col0};
    return plan.parts;
}

int axonn_linear_call_plan(int64_t M, int64_t N, int64_t K, int layout, axonn_plan_part_t parts[AXONN_MAX_PLAN_PARTS]) {
    if (M <= 0 || N <= 0 || K < 0 || layout < 0 || layout > 2 || !parts) return AXONN_ERR_INVALID_ARG;
    axonn::Plan plan = axonn::cached_plan(M, N, K, layout, axonn::g_split_k_enabled.load(std::memory_order_relaxed) != 0);
    if (const size_t need = axonn::split_bytes(plan))
        if (!axonn::registered_scratch(need).partials) plan = axonn::cached_plan(M, N, K, layout, false);
    for (int i = 0; i < plan.parts; ++i)
        parts[i] = axonn_plan_part_t{plan.part[i].variant, plan.part[i].m, plan.part[i].n, plan.part[i].row0, plan.part[i].col0};
    return plan.parts;
}

int axonn_linear_init(void) {
    axonn::raise_lds_limits_once();
    return axonn::static_scratch().partials ? AXONN_OK : AXONN_ERR_WORKSPACE;
}

size_t axonn_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int layout) {
    if (M <= 0 || N <= 0 || K <= 0 || layout < 0 || layout > 2) return 0;
    const size_t bytes = axonn::split_bytes(axonn::cached_plan(M, N, K, layout, true));
    // never less than what axonn_linear_set_workspace accepts (a plan of 128 x 128 tiles can need less)
    return bytes ? axonn::kFlagBytes + std::max(bytes, axonn::kSlotBytes) : 0;
}

int axonn_linear_set_workspace(void* dev_ptr, size_t bytes) {
    if ((dev_ptr == nullptr) != (bytes == 0) || (reinterpret_cast<uintptr_t>(dev_ptr) & 255)) return AXONN_ERR_INVALID_ARG;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= axonn::kMaxDevices) return AXONN_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(axonn::g_scratch_mutex);
    axonn::Scratch& sc = axonn::g_scratch[dev];
    if (dev_ptr == nullptr) {            // unregistered: from now on the kernels that need no scratch
        sc = axonn::Scratch{};
        return AXONN_OK;
    }
    if (bytes < axonn::kFlagBytes + axonn::kSlotBytes) return AXONN_ERR_WORKSPACE;
    // flags start at zero (a flag is valid when it equals the launch's non-zero epoch)
    if (hipMemset(dev_ptr, 0, axonn::kFlagBytes) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        (void)hipGetLastError();
        return AXONN_ERR_WORKSPACE;
    }
    sc = axonn::carve(dev_ptr, bytes);
    return AXONN_OK;
}

int axonn_linear_set_split_k(int enable) {
    if (enable != 0 && enable != 1) return AXONN_ERR_INVALID_ARG;
    return axonn::g_split_k_enabled.exchange(enable, std::memory_order_relaxed);
}

int axonn_linear_split_k_timeouts(uint64_t* count) {
    if (!count) return AXONN_ERR_INVALID_ARG;
    *count = 0;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= axonn::kMaxDevices) return AXONN_ERR_LAUNCH;
    uint32_t* counters[2] = {nullptr, nullptr};   // the registered area's and the static area's
    {
        std::lock_guard<std::mutex> lock(axonn::g_scratch_mutex);
        if (axonn::g_scratch[dev].flags) counters[0] = axonn::g_scratch[dev].timeouts();
    }
    {
        std::lock_guard<std::mutex> lock(axonn::g_static_mutex);
        if (axonn::g_static_ptr[dev]) counters[1] = axonn::carve(axonn::g_static_ptr[dev], axonn::kStaticBytes).timeouts();
    }
    for (uint32_t* counter : counters) {
        if (!counter) continue;   // no split-K kernel has used that area on this device
        uint32_t v = 0;
        if (hipMemcpy(&v, counter, sizeof v, hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError();
            return AXONN_ERR_LAUNCH;
        }
        *count += v;
    }
    return AXONN_OK;
}

int axonn_transpose_bf16(int64_t rows, int64_t cols, const void* src, void* dst, void* stream) {
    constexpr int64_t kMaxDim = (int64_t)1 << 31, kMaxElems = (int64_t)1 << 40;
    if (rows < 0 || cols < 0 || rows >= kMaxDim || cols >= kMaxDim || rows * cols >= kMaxElems) return AXONN_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return AXONN_OK;
    const uintptr_t s = reinterpret_cast<uintptr_t>(src), d = reinterpret_cast<uintptr_t>(dst);
    const uintptr_t bytes = (uintptr_t)rows * (uintptr_t)cols * 2;
    if (!src || !dst || (s & 1) || (d & 1) || (s < d + bytes && d < s + bytes)) return AXONN_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    if (rows % axonn::TR_TILE == 0 && cols % axonn::TR_TILE == 0 && !(s & 15) && !(d & 15)) {
        const int64_t tiles = (rows / axonn::TR_TILE) * (cols / axonn::TR_TILE);
        if (tiles >= kMaxDim) return AXONN_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(axonn::transpose_tile_kernel, dim3((unsigned)tiles), dim3(256), 0, st,
                           static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), rows, cols,
                           (int)(cols / axonn::TR_TILE));
    } else {
        const dim3 grid((unsigned)((rows + 63) / 64), (unsigned)((cols + 3) / 4));
        if (grid.y > 65535u) return AXONN_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(axonn::transpose_naive_kernel, grid, dim3(256), 0, st, static_cast<const uint16_t*>(src),
                           static_cast<uint16_t*>(dst), rows, cols);
    }
    return hipGetLastError() == hipSuccess ? AXONN_OK : AXONN_ERR_LAUNCH;
}

static bool comm_args_ok(const int* grid, int g_node, double beta_inter, double bytes_per_element) {
    if (!grid || g_node < 1 || !(beta_inter > 0.0) || !(bytes_per_element > 0.0)) return false;
    for (int i = 0; i < 4; ++i)
        if (grid[i] < 1) return false;
    return true;
}

int axonn_comm_group_bandwidths(const int* grid, int g_node, double beta_inter, const double* intra_bw, double* beta_out) {
    if (!comm_args_ok(grid, g_node, beta_inter, 1.0) || !beta_out) return AXONN_ERR_INVALID_ARG;
    return axonn::comm_group_bandwidths(grid, g_node, beta_inter, intra_bw, beta_out) ? AXONN_OK : AXONN_ERR_INVALID_ARG;
}

int axonn_comm_layer_time(const axonn_comm_layer_t* layer, const int* grid, const double* beta, double bytes_per_element,
                          double* terms_out) {
    if (!layer || !beta || !terms_out || !comm_args_ok(grid, 1, 1.0, bytes_per_element)) return AXONN_ERR_INVALID_ARG;
    if (layer->m < 0 || layer->k < 0 || layer->n < 0) return AXONN_ERR_INVALID_ARG;
    for (int i = 0; i < 4; ++i)
        if (grid[i] > 1 && !(beta[i] > 0.0)) return AXONN_ERR_INVALID_ARG;
    axonn::comm_layer_terms(*layer, grid, beta, bytes_per_element, terms_out);
    return AXONN_OK;
}

int64_t axonn_comm_rank_grids(int64_t g_total, const axonn_comm_layer_t* layers, int n_layers, int g_node,
                              double beta_inter, const double* intra_bw, double bytes_per_element,
                              axonn_comm_grid_t* out, int64_t max_out) {
    const int one[4] = {1, 1, 1, 1};
    if (g_total < 1 || g_total > ((int64_t)1 << 30) || n_layers < 0 || (n_layers > 0 && !layers) || max_out < 0 ||
        (max_out > 0 && !out) || !comm_args_ok(one, g_node, beta_inter, bytes_per_element))
        return AXONN_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l)
        if (layers[l].m < 0 || layers[l].k < 0 || layers[l].n < 0) return AXONN_ERR_INVALID_ARG;
    std::vector<int64_t> divs;
    for (int64_t d = 1; d * d <= g_total; ++d)
        if (g_total % d == 0) {
            divs.push_back(d);
            if (d != g_total / d) divs.push_back(g_total / d);
        }
    std::sort(divs.begin(), divs.end());
    std::vector<axonn_comm_grid_t> rows;
    for (int64_t gx : divs)
        for (int64_t gy : divs) {
            if ((g_total / gx) % gy) continue;
            const int64_t r2 = g_total / gx / gy;
            for (int64_t gz : divs) {
                if (r2 % gz) continue;
                const int grid[4] = {(int)gx, (int)gy, (int)gz, (int)(r2 / gz)};
                double beta[4], terms[6], total = 0.0;
                if (!axonn::comm_group_bandwidths(grid, g_node, beta_inter, intra_bw, beta)) return AXONN_ERR_INVALID_ARG;
                for (int l = 0; l < n_layers; ++l) {
                    axonn::comm_layer_terms(layers[l], grid, beta, bytes_per_element, terms);
                    total += terms[5];
                }
                rows.push_back(axonn_comm_grid_t{grid[0], grid[1], grid[2], grid[3], total});
            }
        }
    std::sort(rows.begin(), rows.end(), [](const axonn_comm_grid_t& a, const axonn_comm_grid_t& b) {
        if (a.seconds != b.seconds) return a.seconds < b.seconds;
        if (a.gx != b.gx) return a.gx < b.gx;
        if (a.gy != b.gy) return a.gy < b.gy;
        if (a.gz != b.gz) return a.gz < b.gz;
        return a.gdata < b.gdata;
    });
    const int64_t n_out = std::min<int64_t>(max_out, (int64_t)rows.size());
    for (int64_t i = 0; i < n_out; ++i) out[i] = rows[i];
    return (int64_t)rows.size();
}

int axonn_linear_force_variant(int variant) {
    if (variant < -1 || variant >= axonn::num_variants()) return AXONN_ERR_INVALID_ARG;
    axonn::g_forced.store(variant, std::memory_order_relaxed);
    return AXONN_OK;
}

}  // extern "C"
