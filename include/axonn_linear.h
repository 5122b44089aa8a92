/*
 * axonn_linear -- the per-GPU matrix multiplies of a tensor-parallel FC layer
 * on AMD MI355X (CDNA4, gfx950), as a plain C ABI.
 *
 * An FC layer performs one half-precision matrix multiply in the forward pass
 * and two in the backward pass (paper Sec. IV-A, paragraph introducing the
 * three multiplies; Algorithm 1 lines 3, 11 and 13):
 *
 *     forward           O      = I     x W        axonn_linear_fwd
 *     backward, data    dL/dI  = dL/dO x W^T      axonn_linear_bwd_data
 *     backward, weight  dL/dW  = I^T   x dL/dO    axonn_linear_bwd_weight
 *
 * Each call is  C[M,N] = sum over k < K of a(i,k) * b(k,j)  with bf16 operands,
 * fp32 accumulation over the whole K range and one round-to-nearest-even
 * conversion to bf16 at the store.  M, N, K are the dimensions of THIS product
 * (output M x N, reduction length K), not of the layer.
 *
 * `layout` is the mode of Sec. IV-C (NN, NT, TN), in row-major terms, first
 * letter = first operand:
 *
 *     AXONN_NN   first is [M,K], second is [K,N]     C = A   * B
 *     AXONN_NT   first is [M,K], second is [N,K]     C = A   * B^T
 *     AXONN_TN   first is [K,M], second is [K,N]     C = A^T * B
 *
 * (A column-major BLAS names the same three storage patterns NN, TN and NT.)
 * With the buffers the method keeps from the forward pass -- I as [tokens,in],
 * W as [in,out], dL/dO as [tokens,out] -- the natural calls are
 *     fwd       (tokens, out, in,     AXONN_NN, I,     W,     O )
 *     bwd_data  (tokens, in,  out,    AXONN_NT, dL/dO, W,     dL/dI)
 *     bwd_weight(in,     out, tokens, AXONN_TN, I,     dL/dO, dL/dW)
 * and the other six (function, layout) pairs expect the caller to hold a
 * transposed copy of one operand.
 *
 * Common rules for the three entry points
 *   pointers   DEVICE pointers to bf16 (16-bit) elements, row-major, tightly
 *              packed, 16-byte aligned.  The caller owns all three buffers; the
 *              library keeps no reference after return and never reads the
 *              output.  The output must not overlap an input.
 *   scratch    outputs of few tiles and long K are computed fastest by split-K kernels,
 *              which exchange fp32 partial tiles through a scratch area.  The library
 *              allocates NO device memory: the area is memory of the caller's,
 *              registered per GPU with axonn_linear_set_workspace (size it with
 *              axonn_linear_workspace_bytes; 4 KiB + 64 MiB covers every product).
 *              Without a registered area, or for a product that needs a larger one,
 *              the kernels that need no scratch run (same result to the last bit is
 *              NOT promised between the two: the summation order differs).
 *              Calls that may EXECUTE CONCURRENTLY on one GPU (different streams)
 *              would share the area and corrupt each other's partial sums: serialise
 *              them or switch split-K off (axonn_linear_set_split_k).  Calls on one
 *              stream are always safe.
 *   stream     a hipStream_t passed as void*; NULL is the default stream.  The
 *              call enqueues work and returns; it never synchronises and never
 *              allocates, so it may be captured into a HIP graph and replayed.
 *   fp32_accumulate
 *              1: fp32 accumulators over all of K, one rounding at the store.
 *              0: the caller does not require fp32; the same kernels run (the
 *              bf16 matrix instructions of CDNA4 accumulate in fp32 anyway), so
 *              0 is never less accurate than 1.  Other values: INVALID_ARG.
 *   sizes      M, N, K >= 0, each below 2^31, and each operand below 2^40 elements.
 *              M == 0 or N == 0: nothing to do, AXONN_OK.  K == 0: the output is
 *              set to +0.  Any M, N, K is computed correctly; the fast tiled
 *              kernels need M and N to be multiples of 128 and K of 32 (K >= 160).  Other
 *              shapes take a slower guarded MFMA kernel: for the whole product if K does
 *              not suit the tiled kernels, else only for the last columns and rows beyond
 *              the whole 128 x 128 tiles.
 *   errors     the return value is AXONN_OK (0) or a negative code below; on an
 *              error nothing has been launched.  No exceptions, no aborts.
 *   threads    callable from any thread; the process-wide state is the kernel
 *              override (axonn_linear_force_variant), the split-K switch and the
 *              scratch area described above.
 *   determinism the same inputs give the same bits on every call: no floating-point
 *              atomics, fixed summation order per kernel variant (split-K adds
 *              the partial tiles in K order).
 */
#ifndef AXONN_LINEAR_H
#define AXONN_LINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { AXONN_NN = 0, AXONN_NT = 1, AXONN_TN = 2 } axonn_layout_t;

enum {
    AXONN_OK = 0,
    AXONN_ERR_INVALID_ARG = -1, /* null / misaligned pointer, negative or oversized dim, bad enum or flag */
    AXONN_ERR_UNSUPPORTED = -2, /* a forced kernel variant cannot run this shape */
    AXONN_ERR_LAUNCH = -3,      /* the HIP runtime refused the launch */
    AXONN_ERR_WORKSPACE = -4    /* a forced split-K variant has no registered scratch area, or too small a one */
};

/* Forward, Algorithm 1 line 3:  Y[M,N] = X * W.  X and W stored as `layout` says. */
int axonn_linear_fwd(int64_t M, int64_t N, int64_t K, int layout,
                     const void *X, const void *W, void *Y,
                     int fp32_accumulate, void *stream);

/* Backward w.r.t. the input, Algorithm 1 line 11:  dX[M,N] = dY * W^T.
 * M = tokens, N = in features, K = out features; dY is the first operand, W the second
 * (AXONN_NT takes W exactly as the forward pass stored it, [in,out] = [N,K]). */
int axonn_linear_bwd_data(int64_t M, int64_t N, int64_t K, int layout,
                          const void *dY, const void *W, void *dX,
                          int fp32_accumulate, void *stream);

/* Backward w.r.t. the weight, Algorithm 1 line 13:  dW[M,N] = X^T * dY.
 * M = in features, N = out features, K = tokens; X is the first operand, dY the second
 * (AXONN_TN takes both exactly as stored, [tokens,in] = [K,M] and [tokens,out] = [K,N]). */
int axonn_linear_bwd_weight(int64_t M, int64_t N, int64_t K, int layout,
                            const void *X, const void *dY, void *dW,
                            int fp32_accumulate, void *stream);

/* For callers that cannot allocate device memory or register a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same product as the three entry
 * points above (which are one function under three names: `first`, `second`, `out` are X, W, Y /
 * dY, W, dX / X, dY, dW), with the split-K kernels exchanging their partial tiles through a scratch
 * area INSIDE the library: a file-scope device array of axonn_linear_static_scratch_bytes() =
 * 4 KiB + 32 MiB that every GPU the library runs on holds from load until the process ends.  The call
 * allocates nothing, frees nothing, synchronises nothing and ignores any registered workspace.
 * Arguments, layouts, results and error codes are those of axonn_linear_fwd; in addition
 *   - a product whose plan needs more than 128 partial tiles of 256 x 256 fp32 (32 MiB; for example
 *     M = N = 2048, K = 32768: four K ranges on 64 tiles = 192 partial tiles) is refused with
 *     AXONN_ERR_WORKSPACE and nothing is launched (use the entry points above with a registered
 *     workspace for those);
 *   - every call on one GPU uses that GPU's one array: calls that may execute concurrently on one GPU
 *     (different streams) race on it; calls on one stream are safe.  The flag words start at zero
 *     (the array is zero-filled at load) and every kernel leaves them at zero; partial tiles are
 *     always written before they are read, so what an earlier call left there does not matter. */
int axonn_linear_gemm_static(int64_t M, int64_t N, int64_t K, int layout,
                             const void *first, const void *second, void *out,
                             int fp32_accumulate, void *stream);
/* Size in bytes of that array (per GPU).  Host only. */
size_t axonn_linear_static_scratch_bytes(void);

/* Operand re-storage for another mode (Sec. IV-C: the three modes differ only in how each operand
 * lies in memory): dst[cols, rows] = transpose of src[rows, cols], bf16 (16-bit) elements, bit
 * patterns moved unchanged.  DEVICE pointers, row-major, tightly packed, 2-byte aligned, not
 * overlapping; the caller owns both.  rows, cols >= 0 (nothing to do when either is 0), each below
 * 2^31.  Shapes that are multiples of 64 with 16-byte aligned pointers take the fast tiled kernel;
 * others a guarded one, which needs cols <= 262140 (else AXONN_ERR_UNSUPPORTED).  Enqueues on
 * `stream` and returns.  AXONN_OK, AXONN_ERR_INVALID_ARG, AXONN_ERR_UNSUPPORTED or
 * AXONN_ERR_LAUNCH; nothing launched on error. */
int axonn_transpose_bf16(int64_t rows, int64_t cols, const void *src, void *dst, void *stream);

/* Mode tuner (Sec. IV-C: time each product in the three modes during the first batch and keep the
 * fastest).  `op` is 0 (fwd), 1 (bwd_data) or 2 (bwd_weight); `first`, `second` are that product's
 * operands stored the way the method caches them, i.e. in its natural mode (fwd NN, bwd_data NT,
 * bwd_weight TN), `out` its [M,N] output (overwritten with the product).  For every mode the call
 * re-stores the operand(s) that mode wants transposed into `scratch` (DEVICE memory, 256-byte
 * aligned, caller-owned; a mode that needs more than `scratch_bytes` is skipped and reports
 * gemm_us = -1; M*K*2 rounded up to 256 plus K*N*2 bytes is enough for all), times the re-storage
 * and the GEMM with events on `stream`, and SYNCHRONISES with the stream.  The result is returned
 * and remembered under (op, M, N, K):
 *   gemm_us[m]            mean time of the product in mode m (AXONN_NN, _NT, _TN), microseconds
 *   restore_first_us[m]   time to re-store the first / second operand for mode m (0 if that mode
 *   restore_second_us[m]  takes it as cached)
 *   best_layout           mode with the smallest gemm_us
 *   best_layout_all_in    mode with the smallest gemm_us + re-storage of the operands that change
 *                         with every call (all but the weight, i.e. but the second operand of fwd
 *                         and bwd_data, which changes once per optimiser step)
 * AXONN_OK, AXONN_ERR_INVALID_ARG or AXONN_ERR_LAUNCH. */
typedef struct {
    int best_layout;
    int best_layout_all_in;
    float gemm_us[3];
    float restore_first_us[3];
    float restore_second_us[3];
} axonn_tune_result_t;
int axonn_linear_tune(int op, int64_t M, int64_t N, int64_t K, const void *first, const void *second, void *out,
                      void *scratch, size_t scratch_bytes, void *stream, axonn_tune_result_t *result);
/* The remembered result for (op, M, N, K): returns 1 and fills *result, 0 if that product has not
 * been tuned in this process, AXONN_ERR_INVALID_ARG on a bad argument.  Host only. */
int axonn_linear_tuned(int op, int64_t M, int64_t N, int64_t K, axonn_tune_result_t *result);
/* Remember `*result` under (op, M, N, K) as if the tuner had measured it (a caller that keeps its
 * tuning results across runs, or a test).  AXONN_OK or AXONN_ERR_INVALID_ARG.  Host only. */
int axonn_linear_tuned_set(int op, int64_t M, int64_t N, int64_t K, const axonn_tune_result_t *result);
/* Forget all remembered results. */
void axonn_linear_tune_reset(void);

/* Run a product in its tuned mode (Sec. IV-C: "keep the fastest for the rest of training").  `op`,
 * `first`, `second`, `out` as for axonn_linear_tune: the operands as the method caches them (natural
 * mode).  The mode is the remembered best_layout_all_in of (op, M, N, K), or the natural mode if the
 * product has not been tuned.  Operands which that mode wants stored the other way:
 *   first             re-stored into `scratch` by this call, on `stream` (it changes with every call);
 *   second            taken from `second_restored` if that is not NULL -- a transposed copy
 *                     ([N,K] for fwd, [K,N] for bwd_data, [N,K] for bwd_weight) that the caller made
 *                     with axonn_transpose_bf16 and keeps up to date, the way to hold a weight (it
 *                     changes once per optimiser step) -- else re-stored into `scratch` by this call.
 * `scratch`: DEVICE memory, 256-byte aligned, caller-owned; M*K*2 rounded up to 256 plus K*N*2 bytes
 * cover every case; if it is too small for what the tuned mode needs, the product runs in its
 * natural mode, which needs none.  *layout_used (may be NULL) receives the mode that ran.  Enqueues
 * on `stream` and returns; allocates nothing.  Return codes of axonn_linear_fwd. */
int axonn_linear_tuned_call(int op, int64_t M, int64_t N, int64_t K,
                            const void *first, const void *second, void *out,
                            const void *second_restored, void *scratch, size_t scratch_bytes,
                            int fp32_accumulate, void *stream, int *layout_used);

/* ---- communication performance model (Sec. IV-B, Eq. 1-7); host only, no GPU is touched -------- */

/* One FC layer: an m x k input batch times a k x n weight (global sizes, before any sharding);
 * transposed != 0 for the layers whose weight is stored 'transposed', for which the X and Y process
 * groups trade places. */
typedef struct {
    int64_t m, k, n;
    int transposed;
} axonn_comm_layer_t;

/* A 4D grid and the modelled communication time of one pass over the layers. */
typedef struct {
    int gx, gy, gz, gdata;
    double seconds;
} axonn_comm_grid_t;

/* Bandwidth (bytes/s) each of the four process groups of grid[4] = {G_x, G_y, G_z, G_data} sees,
 * hierarchy X innermost.  A group that fits in a node of g_node GPUs reads the profiled table
 * intra_bw[inner * (g_node + 1) + size] (inner = product of the inner group sizes, size = own size;
 * (g_node + 1)^2 doubles, entries with inner * size <= g_node and size >= 2 are used); a group
 * spanning nodes gets beta_inter / min(g_node, inner) (Eq. 7).  A group of one GPU gets +infinity.
 * AXONN_OK, or AXONN_ERR_INVALID_ARG (bad sizes, or a needed table entry is missing or <= 0). */
int axonn_comm_group_bandwidths(const int *grid, int g_node, double beta_inter, const double *intra_bw,
                                double *beta_out);

/* Eq. 1-6 for one layer: terms_out[6] = {all-gather_z, reduce-scatter_z, all-reduce_y, all-reduce_x,
 * all-reduce_data, their sum} in seconds, for beta[4] = bandwidths of the X, Y, Z, data groups. */
int axonn_comm_layer_time(const axonn_comm_layer_t *layer, const int *grid, const double *beta,
                          double bytes_per_element, double *terms_out);

/* Every ordered factorisation G_x * G_y * G_z * G_data = g_total, ranked by the summed time over the
 * layers (ties: smaller G_x, then G_y, G_z first).  Writes the best min(max_out, count) grids to
 * `out` and returns the count of all grids, or a negative error code. */
int64_t axonn_comm_rank_grids(int64_t g_total, const axonn_comm_layer_t *layers, int n_layers, int g_node,
                              double beta_inter, const double *intra_bw, double bytes_per_element,
                              axonn_comm_grid_t *out, int64_t max_out);

/* ---- support ---------------------------------------------------------------------------- */

/* Human-readable text for a status code; never NULL; static storage. */
const char *axonn_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int axonn_linear_version(void);

/* Caller-owned split-K scratch.  axonn_linear_workspace_bytes: what the launches the library would
 * make for this problem need (0: none; otherwise at least the 4 KiB + 256 KiB that
 * axonn_linear_set_workspace accepts).  axonn_linear_set_workspace: use `bytes` bytes at the
 * DEVICE pointer `dev_ptr` (256-byte aligned) as the current device's scratch area from now on; the
 * first 4 KiB are cleared (hipMemset, then a device synchronisation: this call is synchronous).  The
 * caller keeps ownership and must keep the memory alive, and untouched, while it is registered;
 * NULL / 0 unregisters it.  A problem whose need exceeds the registered size, and every problem
 * while nothing is registered, runs without split-K.  Must not be called while GEMM calls are in
 * flight on that device.  AXONN_OK, AXONN_ERR_INVALID_ARG, or AXONN_ERR_WORKSPACE if `bytes` cannot
 * hold a single tile (4 KiB + 256 KiB) or the area could not be cleared. */
size_t axonn_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int layout);
int axonn_linear_set_workspace(void *dev_ptr, size_t bytes);

/* Optional set-up for the current device: raises the kernels' LDS limits and looks up the device
 * address of the static scratch array now rather than inside the first call that needs them
 * (hipFuncSetAttribute, hipGetSymbolAddress; no device memory is allocated, nothing is launched).
 * Idempotent.  AXONN_OK, or AXONN_ERR_WORKSPACE if the address look-up failed. */
int axonn_linear_init(void);

/* Allow (1, the default) or forbid (0) the automatic choice of split-K kernels, process-wide.
 * Returns the previous setting, or AXONN_ERR_INVALID_ARG. */
int axonn_linear_set_split_k(int enable);

/* Diagnostics: how many times, in the scratch area now registered on the current device and in its
 * static array together, a split-K workgroup gave up waiting for a partial tile (it waits about a
 * second; this cannot happen unless another workgroup of the same launch died).  Synchronous
 * device-to-host copies.  *count is 0 when neither has been used. */
int axonn_linear_split_k_timeouts(uint64_t *count);

/* Kernel variants.  Variant 0 is the guarded one-thread-per-element kernel that accepts any
 * shape (the library itself uses it for K == 0 only); the last one ("mfma16_edge_128x128") is the
 * guarded MFMA kernel for any M, N, K >= 1; the others are MFMA tile kernels ("_w8": 8 waves,
 * "_sk2" ... "_sk8": split-K over that many workgroups).  Host-only queries: no GPU is touched. */
int axonn_linear_num_variants(void);
/* Name such as "mfma16k64_256x256_w8_sk2"; NULL if `variant` is out of range. */
const char *axonn_linear_variant_name(int variant);
/* 1 if `variant` can run (M,N,K,layout), else 0 (some variants exist for one layout only). */
int axonn_linear_variant_supports(int variant, int64_t M, int64_t N, int64_t K, int layout);
/* The variant the library would pick for ONE launch over the whole output (pure host logic,
 * ignores any override); negative error code on bad arguments. */
int axonn_linear_select_variant(int64_t M, int64_t N, int64_t K, int layout);
/* The launches the library makes for this problem when no variant is forced.  An output whose
 * tiles fill the 256 compute units a whole number of times and then only part of them is cut
 * into two blocks (the second holds the last rows or the last columns), each with the variant
 * that suits it, e.g. the large tile for the first and split-K for the second.  Block i covers
 * rows row0 .. row0+m-1 and columns col0 .. col0+n-1 of the M x N output; the blocks are
 * disjoint and cover it.  A ragged output (M or N not a multiple of 128) whose K suits the tile
 * kernels, and whose rows start on 16-byte boundaries in all three matrices (N, and for TN also M,
 * a multiple of 8), is planned over its whole tiles as above where that pays, and the last columns
 * and the last rows follow as up to two blocks of the guarded MFMA kernel.  Writes parts[0 .. return value - 1] (HOST
 * memory, caller-owned, room for AXONN_MAX_PLAN_PARTS) and returns the number of launches, 1 to
 * AXONN_MAX_PLAN_PARTS; negative error code on bad arguments.  Pure host logic. */
#define AXONN_MAX_PLAN_PARTS 4
typedef struct {
    int variant;
    int64_t m, n, row0, col0;
} axonn_plan_part_t;
int axonn_linear_plan(int64_t M, int64_t N, int64_t K, int layout, axonn_plan_part_t parts[AXONN_MAX_PLAN_PARTS]);
/* The same for a call made NOW on the current device: as axonn_linear_plan unless the plan needs a
 * larger scratch area than the one registered there (or none is registered), in which case it is
 * the plan without split-K that the call would fall back to.  Host logic plus one hipGetDevice. */
int axonn_linear_call_plan(int64_t M, int64_t N, int64_t K, int layout, axonn_plan_part_t parts[AXONN_MAX_PLAN_PARTS]);
/* Override the choice for all later calls in this process; -1 restores automatic selection.
 * Returns AXONN_OK or AXONN_ERR_INVALID_ARG.  For tests, tuning and the benchmark. */
int axonn_linear_force_variant(int variant);

#ifdef __cplusplus
}
#endif
#endif /* AXONN_LINEAR_H */
