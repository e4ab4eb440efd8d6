/*
 * rmsnl - RMSNorm-then-linear for AMD MI355X (gfx950), C ABI.
 *
 * All pointers named X, g, W, Y, Xn, A are DEVICE pointers (HIP global memory on the
 * current device) owned by the caller; the library reads or writes them on the given
 * stream and never frees or keeps them.  `stream` is a hipStream_t passed as void*
 * (NULL = the default stream).  Every entry point only enqueues work and returns; it
 * performs no host synchronisation, with two exceptions: the first call on a device that needs
 * the library's own workspace (and a later one that needs a larger one) allocates it and clears
 * its counters with a synchronous memset (see rl_set_workspace for how to avoid that), and
 * rl_autotune waits for its timing events.  Matrices are dense and row-major:
 *
 *     X [M][K]   activations        g [K]      gain
 *     W [K][N]   weight, N fastest  Y [M][N]   output
 *
 * Element type is selected by rl_dtype and is the same for all arrays of a call:
 * 16-bit types are accumulated in fp32 and rounded once (nearest-even) when stored.
 * Y must not overlap X, g or W.  Pointers must be aligned to 16 bytes.
 *
 * Errors: every function returns an rl_status; nothing throws or aborts.  Argument
 * checks run before the first HIP call.  rl_last_error() returns a thread-local
 * message for the most recent non-OK status on the calling thread.
 */
#ifndef RMSNL_H
#define RMSNL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#pragma GCC visibility push(default)

typedef enum {
    RL_OK = 0,
    RL_ERR_INVALID_ARG = 1,   /* null / misaligned pointer, size < 1 or >= 2^31, bad enum, eps < 0 or not finite */
    RL_ERR_UNSUPPORTED = 2,   /* a forced variant cannot run this shape or type */
    RL_ERR_HIP = 3,           /* a HIP runtime call failed; text in rl_last_error() */
    RL_ERR_WORKSPACE = 4      /* caller-provided workspace too small */
} rl_status;

typedef enum { RL_F16 = 0, RL_BF16 = 1, RL_F32 = 2 } rl_dtype;

typedef enum {
    RL_AUTO = 0,          /* pick by shape: fp32: its matrix-core kernel, or the plain kernel for what that one does not run.  K or N not
                             a multiple of 8 (gated: N not of 16): the plain kernel.  Else GEMV
                             for M = 1 and N < 10240, and for M <= 4 while K N <= 6e6; M <= 64 skinny, and up to M = 1024 while
                             ceil(M / 64) K N <= 1.4e8 (0.9e8 for N > 6144 and M > 128); else the two-kernel tile form, or the
                             fused tile kernel when the workspace has no room for it.  A shape remembered by rl_autotune is
                             tried first */
    RL_GEMV_SPLITK = 1,   /* M <= 16, 16-bit types, no matrix cores: 64 to 512 columns of W per workgroup, K split into slabs over
                             workgroups; up to 4 rows W goes through LDS by direct loads, above that through registers */
    RL_MFMA_SKINNY = 2,   /* 16-bit types, matrix cores, 64 rows per workgroup (M <= 1024: a row block per 64 rows in the same
                             launch), K split over the waves of a workgroup and into 1 to 16 slabs over workgroups; 128
                             columns of W per workgroup, 64 when that leaves half the chip idle */
    RL_MFMA_TILE = 3,     /* 16-bit types, large M: 256x256 (or 128x512) output tiles on matrix cores, one fused kernel; K < 2^22,
                             N < 2^25; a W of 2 GiB or more is addressed row by row */
    RL_NAIVE = 4,         /* any shape and type, slow (no matrix cores, no split over workgroups): fp32 arithmetic for the
                             16-bit types, fp64 accumulation for fp32 */
    RL_MFMA_TILE_PRE = 5, /* M > 64: X (.) g and 1/rms written once by a first kernel (workspace of 2 M K + 4 M bytes),
                             then the tile kernel as a product scaled per row; with few 256x256 tiles the product is
                             split over K into fp32 partials (up to 64 MiB more) that a third kernel adds up */
    RL_MFMA_F32 = 6       /* fp32 only, any M, K % 4 == 0 and N % 4 == 0, W below 4 GiB: matrix cores on fp32 operands
                             (fp32 products and sums, two levels of accumulators), 64 rows x 64 columns per workgroup,
                             K split over its waves and into 1 to 16 slabs over workgroups */
} rl_variant;

/*
 * Fused RMSNorm + MatMul (case-study section: Eq. 1 followed by the MatMul of Fig. 2a, computed in
 * the reordered form of Fig. 2b; one kernel up to M = 64, see rl_variant for larger M):
 *
 *     A_i  = sum_k X[i][k]^2                      (accumulated in the same K loop as B)
 *     B_in = sum_k (X[i][k] * g[k]) * W[k][n]
 *     Y_in = B_in / sqrt(A_i / K + eps)
 *
 * eps is added to the mean square under the root (eps = 0 gives Eq. 1 exactly).
 * An all-zero row with eps = 0 yields NaN, as the definition does.
 * May use the library workspace (see rl_set_workspace): calls that overlap in time on
 * different streams of one device must not both use it (rl_workspace_bytes() > 0).
 */
rl_status rmsnorm_linear(const void* X, const void* g, const void* W, float eps, void* Y,
                         int64_t M, int64_t K, int64_t N, rl_dtype dt, void* stream);

/*
 * rmsnorm_linear for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same launch shapes and
 * the same result, bit for bit, as rmsnorm_linear; the difference is where the split-K kernels keep
 * their arrival counters and fp32 partial sums: in a fixed device array that is part of the library's
 * code object (rl_noalloc_scratch_bytes() = 8 MiB, of which 1280 KiB are counters and partial sums of
 * squares; every device the library runs on holds its own copy until the process ends), never in
 * memory from hipMalloc.  The call allocates nothing, frees nothing and does not synchronise; it
 * ignores rl_set_workspace.  The first call on a device looks the array's address up and enqueues a
 * small kernel on `stream` that zeroes the counters.
 * A shape whose split-K partials do not fit returns RL_ERR_WORKSPACE ("fixed scratch buffer") and
 * launches nothing; the two-kernel tile form, which would need 2 M K bytes, gives way to the one fused
 * tile kernel, which needs none.
 * All calls on a device share that device's array: calls that overlap in time on one device (different
 * streams, or a graph replayed beside another call) race on it and must be ordered by the caller.
 */
rl_status rmsnorm_linear_noalloc(const void* X, const void* g, const void* W, float eps, void* Y,
                                 int64_t M, int64_t K, int64_t N, rl_dtype dt, void* stream);
size_t rl_noalloc_scratch_bytes(void);

/*
 * The fused block, and the gated block on top of it, with this call's own launch options and
 * workspace instead of the process-wide settings (rl_set_variant, rl_set_tuning, rl_set_workspace):
 * for callers with several streams, and for searches over launch shapes (the paper's search over grid
 * dimensions, restricted to this kernel family).  opts == NULL means RL_AUTO with the library's workspace,
 * i.e. exactly rmsnorm_linear / rmsnorm_gated_mlp.  Every field 0 means "automatic"; fields a variant
 * does not have are ignored; a value the variant cannot honour gives RL_ERR_UNSUPPORTED.
 *
 *   struct_size    sizeof(rl_launch_opts), checked
 *   variant        RL_AUTO or a forced variant (then no fallback, as with rl_set_variant)
 *   columns        GEMV: columns of W per workgroup, 64, 128, 256 or 512; skinny: a multiple of 8 up to 128; fp32: 64;
 *                  fused tile kernel: 256 (256 x 256 tiles) or 512 (128 x 512 tiles)
 *   slabs          K slabs: GEMV, skinny and fp32 (1..16), and the product of the two-kernel tile form (1 = unsplit)
 *   waves          fused tile kernel: waves per workgroup, 4 or 8
 *   rem_slabs      two-kernel tile form: K slabs for the tiles left over after the last full round of 256
 *   workspace      DEVICE buffer of workspace_bytes for this call alone (16-byte aligned, its first 256 KiB
 *                  zero before the first call that uses it; the kernels leave them zero), or NULL for the
 *                  library's own or the lent one.  Calls that run at the same time on different streams of one
 *                  device must each bring their own.  Too small for the call: RL_ERR_WORKSPACE, except
 *                  that RL_AUTO gives up the two-kernel tile form for the fused tile kernel.
 *
 * rmsnorm_gated_mlp_ex: interleaved != 0 reads W as rmsnorm_gated_mlp_interleaved does.
 * rl_last_launch reports what the most recent successful call on this thread launched: variant, columns
 * per workgroup (tile kernels: columns of a tile), K slabs (fused tile kernel: waves) and workgroups of its
 * main kernel.
 */
typedef struct {
    size_t struct_size;
    rl_variant variant;
    int columns;
    int slabs;
    int waves;
    int rem_slabs;
    void* workspace;
    size_t workspace_bytes;
} rl_launch_opts;
rl_status rmsnorm_linear_ex(const void* X, const void* g, const void* W, float eps, void* Y,
                            int64_t M, int64_t K, int64_t N, rl_dtype dt, const rl_launch_opts* opts, void* stream);
rl_status rmsnorm_gated_mlp_ex(const void* X, const void* g, const void* W, float eps, void* Y,
                               int64_t M, int64_t K, int64_t H, rl_dtype dt, int interleaved,
                               const rl_launch_opts* opts, void* stream);
rl_status rl_last_launch(rl_variant* variant, int* columns, int* slabs, int* workgroups);

/*
 * Unfused pair, for A/B comparison with the fused call (the two-kernel baseline of
 * Fig. 2a: the normalised intermediate goes through device memory).
 *
 * rmsnorm: Xn[i][k] = X[i][k] * g[k] / sqrt(mean_k X[i][k]^2 + eps), Eq. 1, rounded to dt.
 * matmul:  Y = A . W with A [M][K], same variants and layout rules as rmsnorm_linear.
 */
rl_status rmsnorm(const void* X, const void* g, float eps, void* Xn,
                  int64_t M, int64_t K, rl_dtype dt, void* stream);
rl_status matmul(const void* A, const void* W, void* Y,
                 int64_t M, int64_t K, int64_t N, rl_dtype dt, void* stream);

/*
 * Gated MLP on top of the fused block (the paper's GatedMLP benchmark: two products of the same
 * input run side by side in one kernel, SiLU and the elementwise product applied as its epilogue;
 * here stacked on the RMSNorm prologue, so the normalised input, the two products and the gate
 * never touch device memory):
 *
 *     W [K][2H] = [gate | up], columns [0, H) the gate half, [H, 2H) the up half, row-major
 *     Z = the block above on all 2H columns (not materialised)
 *     Y[i][h] = SiLU(Z[i][h]) * Z[i][H + h],   SiLU(v) = v / (1 + exp(-v)),   Y [M][H]
 *
 * Same pointer, alignment, eps and workspace rules as rmsnorm_linear; H % 8 == 0 for the fast
 * variants.  silu_mul is the separate activation kernel
 * of the unfused baseline: it reads a materialised Z [M][2H] and writes Y [M][H].
 */
rl_status rmsnorm_gated_mlp(const void* X, const void* g, const void* W, float eps, void* Y,
                            int64_t M, int64_t K, int64_t H, rl_dtype dt, void* stream);
rl_status silu_mul(const void* Z, void* Y, int64_t M, int64_t H, rl_dtype dt, void* stream);

/*
 * The same gated block (the paper's GatedMLP benchmark) on a W whose gate and up columns are
 * interleaved in groups of 64, the layout a caller gives its weights once, when it loads them:
 *
 *     Wi [K][2H]: columns 128 j .. 128 j + 63 are the gate columns of outputs 64 j .. 64 j + 63, columns
 *     128 j + 64 .. 128 j + 127 the up columns of the same outputs; H % 64 == 0
 *     Y[i][h] = SiLU(Z_gate[i][h]) * Z_up[i][h] exactly as rmsnorm_gated_mlp computes it
 *
 * A workgroup that owns a run of outputs then reads one contiguous run of columns per row of W, as
 * in the plain block, instead of two runs half as long that lie H columns apart.  The result is the
 * one rmsnorm_gated_mlp gives on the two-halves W (same kernels, only the column a lane fetches
 * differs).  Tuned by rl_autotune_rotating with interleaved != 0, not by rl_autotune.  rl_interleave_gate_up writes Wi from W = [gate | up] (both
 * [K][2H] DEVICE arrays of type dt, 16-byte aligned, not the same buffer), on `stream`.
 */
rl_status rmsnorm_gated_mlp_interleaved(const void* X, const void* g, const void* Wi, float eps, void* Y,
                                        int64_t M, int64_t K, int64_t H, rl_dtype dt, void* stream);
rl_status rl_interleave_gate_up(const void* W, void* Wi, int64_t K, int64_t H, rl_dtype dt, void* stream);

/*
 * Variant control (process-wide).  RL_AUTO is the default; the environment variable
 * RL_VARIANT (auto|gemv|skinny|tile|tile_pre|naive|f32) sets the initial value.  A forced variant that
 * cannot run a shape makes the call return RL_ERR_UNSUPPORTED instead of falling back.
 * rl_last_variant() reports what the most recent successful call on this thread ran.
 */
rl_status rl_set_variant(rl_variant v);
rl_variant rl_get_variant(void);
rl_variant rl_last_variant(void);

/*
 * Launch-shape overrides for tuning sweeps (process-wide, 0 = automatic; they apply to a forced
 * variant only):
 *   n_tile  columns of W per workgroup (GEMV: 64, 128, 256, 512; skinny: a multiple of 8 up to 128;
 *           tile: 256 = 256x256 tiles, 512 = 128x512 tiles),
 *   k_split number of K slabs (split-K factor) of the GEMV and skinny variants; for the tile variant
 *           the waves per workgroup (4 or 8); for the two-kernel tile variant n_tile = 1 makes k_split
 *           (1 to 16) the number of K slabs of its product (1 = no split; otherwise the library splits
 *           when the 256x256 tiles are too few to fill the chip), and n_tile = 2 makes k_split the number
 *           of slabs for the tiles left over after the last full round of 256 (1 = no such split).
 *           For rl_qknorm_attention k_split is the number of splits of the sequence (at least 64 positions each).
 * Values a variant cannot honour give RL_ERR_UNSUPPORTED at the next call.
 */
rl_status rl_set_tuning(int n_tile, int k_split);

/*
 * Normalised-Transformer chain in one kernel (the paper's nTrans benchmark: two normalisations
 * around an elementwise step, three kernels in existing systems):
 *
 *     Y[i][:] = Norm(X[i][:] + alpha (.) Norm(H[i][:] - X[i][:])),   Norm(v) = v / sqrt(mean(v^2) + eps)
 *
 * X, H, Y [M][D] and alpha [D] DEVICE arrays of type dt, row-major, 16-byte aligned; Y may not
 * overlap the inputs.  "Norm" is read as Eq. 1 without a gain (the paper does not say which
 * normalisation the benchmark uses).  fp32 arithmetic, one rounding when stored.  M < 2^31.
 */
rl_status rl_ntrans(const void* X, const void* H, const void* alpha, float eps, void* Y,
                    int64_t M, int64_t D, rl_dtype dt, void* stream);

/*
 * Launch-shape tuner: the schedule half of the paper's search (grid dimensions, and here the K
 * split that stands in for its for-loop dimension), restricted to this library's kernel family;
 * the paper reports that the choice of grid dimensions alone is worth part of its gain.
 *
 * rl_autotune runs every launch shape the library has for the call, generated from the shape
 * (variant x columns per workgroup x every K slab count that leaves each lane group a batch of rows,
 * launches that come out the same timed once; tile shape x waves per workgroup for the tile
 * variant; the two-kernel form with and without its K split) on the caller's own device
 * buffers: two warm-up launches, then `reps` (1..1000) timed ones between HIP events on `stream`.
 * The fastest is remembered for (M, K, N, dt, gated) and used by later RL_AUTO calls of exactly
 * that shape; forced variants are not affected; a tuned shape that finds no room in the workspace
 * gives way to the built-in one.  `gated` != 0 tunes rmsnorm_gated_mlp (N = 2H, Y is
 * [M][H]), else rmsnorm_linear.  Y is overwritten by every candidate (all compute the same block).
 * This is the one entry point that synchronises with the stream (it waits on its events); it
 * times on the buffers as they are, so a W that fits the 256 MB last-level cache is timed warm.
 * *best_us (may be NULL) receives the winner's time per launch in microseconds.
 * rl_autotune_get reports the remembered choice (variant RL_AUTO if there is none);
 * rl_autotune_clear forgets everything.
 */
rl_status rl_autotune(const void* X, const void* g, const void* W, float eps, void* Y,
                      int64_t M, int64_t K, int64_t N, rl_dtype dt, int gated, int reps,
                      void* stream, float* best_us);
/*
 * The same search on cold data: the timed launches rotate through n_copies DEVICE copies of W
 * (W_copies: host array of n_copies device pointers; enough of them that they exceed the 256 MB
 * last-level cache, e.g. ceil(512 MiB / bytes of W)), so a small W is timed as it comes from HBM and
 * not as it lies in the cache (where more, smaller slabs look better than they are).  interleaved != 0
 * (with gated != 0) tunes rmsnorm_gated_mlp_interleaved on copies of Wi.  The choice is remembered per
 * (M, K, N, dt, gated, interleaved); rl_autotune_get's `gated` takes 1 for the two-halves layout and 3
 * for the interleaved one.
 */
rl_status rl_autotune_rotating(const void* X, const void* g, const void* const* W_copies, int n_copies, float eps, void* Y,
                               int64_t M, int64_t K, int64_t N, rl_dtype dt, int gated, int interleaved, int reps,
                               void* stream, float* best_us);
rl_status rl_autotune_get(int64_t M, int64_t K, int64_t N, rl_dtype dt, int gated,
                          rl_variant* variant, int* n_tile, int* k_split);
void rl_autotune_clear(void);

/*
 * QKNorm in front of attention (the paper's QKNorm benchmark: layer normalisation of the query and key
 * vectors before attention, in one kernel with the attention), decode form: one query per (sample,
 * head) against S cached positions.  DEVICE arrays, row-major: Q [B][H][D], K and V [B][H][S][D],
 * gq, bq, gk, bk [D] (gain and bias of the two layer normalisations, shared by the heads), O [B][H][D]:
 *
 *     LayerNorm(v; g, b)_d = (v_d - mean(v)) / sqrt(var(v) + eps) * g_d + b_d      (population variance)
 *     qn = LayerNorm(q; gq, bq),  kn_t = LayerNorm(k_t; gk, bk),  s_t = qn . kn_t / sqrt(D)
 *     O = sum_t softmax(s)_t v_t
 *
 * The paper names the operation but not its constants: the usual layer normalisation, the usual
 * 1/sqrt(D), eps as given.  Fast path: D = 64, 128 or 256 and a 16-bit type (keys read once, their mean,
 * variance and dot product from the same registers, online softmax, the sequence split over workgroups); any
 * other D (<= 4096) or type, and S D >= 2^30, runs a slow plain kernel.  May use the library workspace like
 * rmsnorm_linear.  Pointers 16-byte aligned; O must not overlap the inputs.
 */
rl_status rl_qknorm_attention(const void* Q, const void* K, const void* V, const void* gq, const void* bq,
                              const void* gk, const void* bk, float eps, void* O,
                              int64_t B, int64_t H, int64_t S, int64_t D, rl_dtype dt, void* stream);

/*
 * The tuner for rl_qknorm_attention (the paper's search over grid dimensions, for this kernel: how many
 * workgroups share a (sample, head)'s sequence).  Times the library's own rule and every number of
 * sequence splits that leaves a split at least 64 positions (counts that come out the same launched once),
 * two warm-up launches and `reps` (1..1000) timed ones each, between HIP events on `stream`, rotating
 * through n_copies DEVICE copies of K and V (host arrays of device pointers; one copy times the cache-warm
 * case).  The fastest is remembered for (B H, S, D, dt) and used by later rl_qknorm_attention calls of that
 * shape unless rl_set_tuning forces a count; rl_autotune_clear forgets it.  *best_splits (may be NULL)
 * receives the number of splits chosen, *best_us its time per launch.  Shapes that run the plain kernel have
 * nothing to search: RL_OK, *best_splits = 0.  O is overwritten by every candidate.  Synchronises with the
 * stream (it waits on its events).
 */
rl_status rl_autotune_qknorm(const void* Q, const void* const* K_copies, const void* const* V_copies, int n_copies,
                             const void* gq, const void* bq, const void* gk, const void* bk, float eps, void* O,
                             int64_t B, int64_t H, int64_t S, int64_t D, rl_dtype dt, int reps, void* stream,
                             int* best_splits, float* best_us);

/*
 * The block over a prime field, for the paper's way of certifying a rewrite (random tests over
 * finite fields, Table 3: add, mul, div and sqrt as modular operations): X [M][K], g [K], W [K][N],
 * Y [M][N] are DEVICE arrays of uint32 with entries in [0, p), p a prime in [3, 32749] that does not
 * divide K.  reordered = 0 evaluates Eq. 1 and then the product (Fig. 2a); reordered = 1 the
 * rewritten graph (Fig. 2b: product first, division by the root afterwards).  Equal outputs on
 * random inputs certify the reordering with the paper's error bound.  sqrt is the canonical root
 * (smallest y with y^2 = x; for a non-residue x the smallest y with y^2 = x n, n the least
 * non-residue); a row whose mean square is 0 gets 0 in both forms.  Integer arithmetic only:
 * results are exact and equal, bit for bit, to the reference evaluation.
 */
rl_status rl_ff_rmsnorm_linear(const void* X, const void* g, const void* W, void* Y,
                               int64_t M, int64_t K, int64_t N, uint32_t p, int reordered, void* stream);

/*
 * The paper's random tests in full (Table 3 with its Exp row; Theorems 2 and 3): the block, and the
 * gated block with its exponential (SiLU), evaluated on PAIRS (x_p, x_q) over Z_p x Z_q with the primes
 * of the paper's implementation, p = 227 and q = 113 (q divides p - 1).  X [M][K], g [K], W [K][N] and Y
 * are DEVICE arrays of uint16, an element being x_p | x_q << 8 (x_p < 227, x_q < 113); 16-byte aligned.
 * Add, Mul, Div and Sqrt act on both components (sqrt: the canonical root of rl_ff_rmsnorm_linear; a
 * row whose mean square is 0 in a field gets 0 there); Exp maps a pair to omega^{x_q} mod p, with omega
 * a q-th root of unity of Z_p that the caller samples, and leaves a p component only.
 *   gated = 0: Y [M][N] pairs, the block.   gated = 1: N = 2H, W = [gate | up], Y [M][H] = G / (1 +
 *   exp(-G)) * U in Z_p (q component 0; 0 where 1 + exp(-G) has no inverse).
 *   schedule = 0: the graph as the paper starts from it -- Eq. 1 first, then the product, then the
 *   activation -- one thread per output.
 *   schedule = 1: the GEMV split-K kernel that rmsnorm_linear and rmsnorm_gated_mlp run, instantiated on
 *   this element type: same column tiles, K slabs (`slabs`, 0 = the kernel's own choice), reduction
 *   through LDS, partials in the workspace added by the last arriver in slab order, same pairing of
 *   gate and up columns, same rewrite (division after the product).  M <= 16, K % 8 == 0, N % 8 == 0
 *   (gated: N % 16 == 0), else RL_ERR_UNSUPPORTED.
 * Equal outputs of the two schedules on random inputs certify the shipped schedule against the graph
 * with the error bound of the paper's theorems; integer arithmetic throughout, results are exact.
 * Neither 227 nor 113 may divide K.
 */
rl_status rl_ff_pairs(const void* X, const void* g, const void* W, void* Y, int64_t M, int64_t K, int64_t N,
                      uint32_t omega, int gated, int schedule, int slabs, void* stream);

/*
 * Workspace (split-K partial sums + arrival counters; X (.) g, 1/rms and partial tiles of the two-kernel
 * tile form, split merges of rl_qknorm_attention).  By default the library allocates
 * rl_workspace_default_bytes() per device on first need and switches to a larger allocation (at least
 * twice the size, up to 4 GiB) when a call needs more; earlier allocations stay alive until the process
 * ends, because a graph captured before still points into them.  Nothing is allocated while the call's
 * stream is being captured into a graph: run the shape once before capturing, or lend a buffer.  rl_set_workspace lends a
 * caller-owned DEVICE buffer instead (for the current device; the first 256 KiB must be zero when lent);
 * NULL returns to the library's own buffer.  With a lent buffer too small for a call, the split-K variants
 * return RL_ERR_WORKSPACE; the two-kernel tile form is then skipped by RL_AUTO (the fused tile kernel runs).
 * rl_workspace_bytes gives the bytes an rmsnorm_linear call of that shape would like (0 if none).
 */
rl_status rl_set_workspace(void* dev_ptr, size_t bytes);
size_t rl_workspace_bytes(int64_t M, int64_t K, int64_t N, rl_dtype dt);
size_t rl_workspace_default_bytes(void);

/*
 * Stage trace (diagnostics).  While a DEVICE buffer is registered, thread 0 of workgroup b of
 * the split-K kernel stores the 100 MHz constant clock into 64-bit slot b*rl_trace_slots()+i
 * when it reaches stage i (0 start, 1 first loads issued, 2 K loop done, 3 workgroup partial
 * reduced, 4 partials published, 5 counter bumped, 6 all slabs read, 7 Y stored); workgroups
 * beyond bytes / (8 * rl_trace_slots()) are not traced.  NULL switches it off (the default).
 * The buffer is caller-owned and must outlive every traced call.
 */
rl_status rl_set_trace(void* dev_ptr, size_t bytes);
size_t rl_trace_slots(void);

/*
 * Launch order of the tile kernels (diagnostics, host only, no device work): the workgroup at
 * `position` (0 .. tiles - 1, tiles = ceil(M / 256) * ceil(N / 256)) of a launch over an M x N output
 * computes the 256 x 256 tile (*tile_row, *tile_col).  The order places the tiles that one XCD runs
 * together in blocks of 4 x 8; every tile appears at exactly one position.  RL_ERR_INVALID_ARG for a
 * position outside the range or more than 2^24 tiles.
 */
rl_status rl_tile_order(int64_t M, int64_t N, int64_t position, int64_t* tile_row, int64_t* tile_col);

/*
 * Measurement helpers (not on the hot path): a plain device-to-device copy kernel of
 * `bytes` bytes (multiple of 16) used to calibrate memory counters and to measure the
 * achievable streaming rate, and a register-only matrix-core loop of `iters` iterations
 * per wave that reports the achievable MFMA rate (writes one float per lane to `sink`,
 * which must hold rl_probe_mfma_sink_floats() floats).  The loop's operands are pseudo-random values
 * in (-2, 2); rl_probe_mfma_operands with zero_operands != 0 runs it on zeros: the matrix cores draw
 * less power without switching activity and the clock stays up, so the two rates bracket what the
 * multipliers allow on real data and what the published peak assumes.
 */
rl_status rl_probe_copy(void* dst, const void* src, size_t bytes, void* stream);
rl_status rl_probe_read(const void* src, size_t bytes, void* sink, void* stream);
rl_status rl_probe_mfma(void* sink, int iters, rl_dtype dt, void* stream);
rl_status rl_probe_mfma_operands(void* sink, int iters, rl_dtype dt, int zero_operands, void* stream);
/*
 * Streaming reads in the launch shapes of the small-M kernels, for a measured ceiling beside their
 * figures.  rl_probe_read_strips: the DEVICE matrix src [rows][row_bytes] (row_bytes a multiple of 256,
 * (rows + 256) * row_bytes < 2^31) is read as the GEMV and skinny kernels read W: one workgroup per
 * 256-byte column strip and row part (`parts` of them, 1 <= parts <= rows), a wave-wide 16-byte load
 * covering 4 rows of 256 bytes.  rl_probe_read_flat: `workgroups` workgroups read contiguous shares of
 * `bytes` bytes, 1 KiB per wave-wide load.  Both read every byte once and write nothing
 * (`sink`: 4 bytes of DEVICE memory that are practically never written).  While a stage trace is
 * registered (rl_set_trace), workgroup b of the strips probe stamps slot 0 when it starts and slot 2
 * when its rows have arrived; its strip is b / parts after the renumbering
 * b -> (b mod 8) * (workgroups / 8) + b / 8 that applies when the workgroups divide by 8.
 */
rl_status rl_probe_read_strips(const void* src, int64_t rows, int64_t row_bytes, int parts, void* sink, void* stream);
rl_status rl_probe_read_flat(const void* src, size_t bytes, int workgroups, void* sink, void* stream);
size_t rl_probe_mfma_sink_floats(void);
double rl_probe_mfma_flops(int iters);

const char* rl_last_error(void);
const char* rl_version(void);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif /* RMSNL_H */
