/*
 * dla.h - C ABI of the MI355X (gfx950) dense linear-algebra kernels that the
 * paper's autotuner compiles and times: 3mm, LU without pivoting, Cholesky
 * (paper, Section "Linear Algebra Benchmarks").
 *
 * Conventions that hold for every entry point
 *   - Matrices are ROW-MAJOR (the paper's X[i, j] indexing in the 3mm
 *     tensor-expression listing); a leading dimension is counted in elements
 *     and must be >= the number of columns.
 *   - Every pointer whose name starts with d_ is a DEVICE pointer owned by the
 *     caller.  The library never allocates or frees caller-visible memory and
 *     keeps no pointer after the call returns.  Scratch memory comes in
 *     through an explicit workspace argument whose size the matching
 *     *_workspace_bytes() query returns.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it asynchronously; no entry point synchronises
 *     the device.  With lookahead enabled a factorisation also uses three
 *     library-owned helper streams that are fork/joined to hip_stream with
 *     events, so from the caller's side the call still behaves as one piece of
 *     work on hip_stream.  Some of its kernels are then launched before the
 *     kernel they depend on has finished and wait for it on counters in the
 *     workspace (a bounded poll), so two factorisations must not share one
 *     workspace while either is still running.  The helper streams and their
 *     events are shared by all calls of the process; a process-wide lock is held
 *     while a factorisation enqueues its work, so calls from several host
 *     threads are safe (each with a workspace of its own) and run one behind the
 *     other on the helper streams.  The profiling switches are not thread safe.
 *   - Return value: DLA_SUCCESS (0); -i when the i-th argument (1-based) is
 *     invalid (null pointer, negative size, leading dimension too small,
 *     unknown dtype, misaligned pointer); or one of the positive DLA_ERR_*
 *     codes.  Argument errors are detected before any GPU work is enqueued.
 *   - Tile sizes, block sizes and unroll factors are explicit parameters (the
 *     paper's split factors P0..P5 of the 3mm code mold and the two tile
 *     parameters of LU/Cholesky) so that a search can drive them.  Only
 *     combinations from a pre-instantiated menu are legal; anything else
 *     returns DLA_ERR_UNSUPPORTED_PARAMS instead of running a slow path.
 *     Tiles need not divide the matrix dimensions.
 */
#ifndef DLA_H
#define DLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DLA_F64 = 0, DLA_F32 = 1 } dla_dtype;

enum {
  DLA_SUCCESS = 0,
  DLA_ERR_UNSUPPORTED_PARAMS = 1, /* tile/block combination not in the menu          */
  DLA_ERR_WORKSPACE = 2,          /* workspace missing, misaligned or too small        */
  DLA_ERR_HIP = 3,                /* a HIP call or kernel launch failed                */
  DLA_ERR_TOO_LARGE = 4           /* a dimension exceeds what the kernels index (2^31) */
};

/* Kernel selectors for dla_default_params(). */
enum { DLA_KERNEL_MM3 = 0, DLA_KERNEL_LU = 1, DLA_KERNEL_CHOLESKY = 2 };

/*
 * Schedule of one GEMM.  tile_m x tile_n is the macro-tile one workgroup
 * computes: the paper's split factors of the y and x axes of one 3mm product
 * (code mold, parameters P0..P5).  The remaining fields are the extra knobs of
 * the native kernel.  A field set to 0 means "library default for this
 * macro-tile".
 */
typedef struct {
  int tile_m, tile_n; /* workgroup macro-tile, multiples of 16                                 */
  int tile_k;         /* depth of the k-slab staged in LDS per main-loop iteration (8/16/32/128) */
  int unroll_k;       /* 16x16x4 MFMA k-steps unrolled together inside a slab (1, 2, 4, 8)      */
  int wave_m, wave_n; /* sub-tile one 64-lane wavefront accumulates in registers                */
} dla_gemm_params;

/*
 * Schedule of a blocked right-looking factorisation.  nb is the panel width
 * (block size), update the schedule of the trailing-matrix update
 * A22 -= L21 * U12 (lower(A22) -= L21 * L21^T for Cholesky) that dominates the run time:
 * all six fields 0 (the default) selects the
 * library's panel-stationary rank-nb update kernel; if any field is set the
 * update runs as tiled GEMMs with that schedule (fields left 0 take the menu's
 * defaults), so that a search can drive each of them.
 *
 * Block sizes.  16 .. 128 in steps of 16: one level of blocking, the diagonal block is factored by one
 * workgroup out of LDS (128 x 128 fp64 is what fits).  160, 192, 224, 256: two levels.  The panel of nb
 * columns is factored as two sub-panels of nb / 2, and the bulk of the trailing matrix receives both
 * at once in one update of depth nb (twice the flops per byte of the trailing matrix); these need the
 * look-ahead pipeline and the default update kernel, otherwise DLA_ERR_UNSUPPORTED_PARAMS.  With
 * nb = 128 the same two-level form (depth 256, sub-panels of 128) is used on its own accord while the
 * trailing matrix is large; defer_min_rows moves that threshold.
 *
 * There is no separate inner block size of the diagonal-block kernel: it works in stages of 16 columns,
 * the edge of the MFMA block, and nothing else is instantiated.
 */
typedef struct {
  int nb;        /* block size (0 = default 128); see above                                     */
  int lookahead; /* 0: one stream, strictly sequential steps; 1: the next diagonal block is factored
                    while panel solves and trailing update of this step run on helper streams, and
                    the kernels of that chain wait for each other inside the kernels (needs kernels
                    of the process to run side by side); 2: the same pipeline ordered by stream
                    events only, for tools that serialise kernels (hardware-counter profiling,
                    debuggers); -1 = default (1)                                                */
  dla_gemm_params update;
  int defer_min_rows; /* nb = 128 only: bulk updates run two panels deep while the trailing matrix has
                         at least this many rows.  0 = library default (2560; 4096 for fp32 Cholesky),
                         -1 = never, 1 = whenever possible.  Ignored for other block sizes.      */
} dla_factor_params;

/* The six tile parameters of the 3mm code mold: (P0,P1) -> e, (P2,P3) -> f, (P4,P5) -> g. */
typedef struct {
  dla_gemm_params e, f, g;
} dla_mm3_params;

/*
 * LU decomposition without pivoting, A = L*U, in place (paper, Section
 * "Linear Algebra Benchmarks": L lower, U upper, no pivoting).
 *   d_a        device, n x n, row-major with leading dimension lda; on exit the
 *              strict lower triangle holds L (unit diagonal not stored) and the
 *              upper triangle including the diagonal holds U.
 *   p          schedule, or NULL for defaults.
 *   d_workspace / workspace_bytes   device scratch of at least
 *              factor_workspace_bytes(n, dt, p) bytes, 256-byte aligned.
 *   d_info     device int, may be NULL.  Written asynchronously: 0, or the
 *              1-based index of the first exactly-zero pivot, after which the
 *              content of A is unspecified (the call itself still completes);
 *              or -1: with lookahead = 1 a kernel gave up waiting for its
 *              predecessor (after 0.1 s plus several times the duration of the
 *              call's largest update: kernels of the process do not run side by
 *              side), the content of A is invalid, use lookahead = 2 or 0.
 *              Because that report needs d_info, a call with d_info == NULL and
 *              lookahead = 1 runs as lookahead = 2 (stream events order the
 *              chain; about a tenth slower at N = 4000, never invalid).
 * n == 0 is a successful no-op.
 */
int lu_factor(void* d_a, int64_t n, int64_t lda, dla_dtype dt, const dla_factor_params* p,
              void* d_workspace, size_t workspace_bytes, void* hip_stream, int* d_info);

/*
 * Cholesky decomposition A = L*L^T, in place (same Section).  Only the lower
 * triangle of A (diagonal included) is read.  On exit the lower triangle holds
 * L and the strict upper triangle is zero.  d_info: 0, or the 1-based index of
 * the first pivot that is not strictly positive.  Other arguments as lu_factor.
 */
int cholesky_factor(void* d_a, int64_t n, int64_t lda, dla_dtype dt, const dla_factor_params* p,
                    void* d_workspace, size_t workspace_bytes, void* hip_stream, int* d_info);

/*
 * Solving A*X = B with the factors (paper, Section "Introduction": LU and Cholesky are named as the
 * factorisations behind solving systems of linear equations).  lu_solve: L*Y = B by forward substitution (unit diagonal),
 * then U*X = Y backward.  cholesky_solve: L*Y = B, then L^T*X = Y (only the lower triangle is read).
 *   d_lu / d_l   device, n x n, leading dimension lda: the output of lu_factor / cholesky_factor;
 *                read only.
 *   d_b          device, n x nrhs, row-major with leading dimension ldb (every column is one
 *                right-hand side); overwritten by X.  Must not overlap the factor.
 *   d_workspace / workspace_bytes   device scratch of at least solve_workspace_bytes(n, nrhs, dt)
 *                bytes, 256-byte aligned: per 256 rows of the factor and substitution a 256 x 256
 *                inverted diagonal block and its 256 x 512 product with the factor's blocks beside
 *                it (13 KB per row of the factor in fp64), and two n x nrhs areas for the
 *                solutions of the forward and the backward pass.
 * n == 0 or nrhs == 0 is a successful no-op that needs no workspace.  A zero on the factor's diagonal
 * gives infinities or NaNs in X; nothing is reported (the factorisation's d_info already said so).
 */
int lu_solve(const void* d_lu, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
             void* d_workspace, size_t workspace_bytes, void* hip_stream);
int cholesky_solve(const void* d_l, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
                   void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Scratch bytes lu_solve / cholesky_solve need (same for both). 0 on invalid arguments. */
size_t solve_workspace_bytes(int64_t n, int64_t nrhs, dla_dtype dt);

/*
 * The same solves in two parts, for callers that solve with one factor again and again (paper, Section
 * "Introduction": the factorisations are what solving systems of linear equations is built on).
 * lu_solve_prepare / cholesky_solve_prepare run the part of the solve that does not depend on B (the
 * inverted diagonal blocks and their products with the factor's blocks beside them: 0.12 ms of lu_solve's
 * 0.37 ms at n = 4000 with 64 right-hand sides) and leave it in the workspace; lu_solve_prepared /
 * cholesky_solve_prepared then overwrite B with X like lu_solve / cholesky_solve, bit for bit the same
 * result, from a workspace that the matching prepare call has filled FOR THIS FACTOR (same d_lu / d_l
 * contents, n, lda, dt, same kind) and that nothing else has written since; any number of them may follow
 * one prepare call, with any nrhs the workspace has room for.  A workspace that was not prepared, or was
 * prepared for another factor, gives a wrong X and no error: the library cannot tell.
 *   d_workspace / workspace_bytes   prepare: at least solve_workspace_bytes(n, 0, dt) bytes; prepared: at
 *                least solve_workspace_bytes(n, nrhs, dt) bytes of the SAME allocation (the part the
 *                prepare call filled lies at its start and does not depend on nrhs); 256-byte aligned.
 * Other arguments, order on hip_stream and return codes as for lu_solve / cholesky_solve (negative: the
 * position of the offending argument).  n == 0 is a successful no-op, as is nrhs == 0.
 */
int lu_solve_prepare(const void* d_lu, int64_t n, int64_t lda, dla_dtype dt, void* d_workspace, size_t workspace_bytes,
                     void* hip_stream);
int cholesky_solve_prepare(const void* d_l, int64_t n, int64_t lda, dla_dtype dt, void* d_workspace,
                           size_t workspace_bytes, void* hip_stream);
int lu_solve_prepared(const void* d_lu, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
                      void* d_workspace, size_t workspace_bytes, void* hip_stream);
int cholesky_solve_prepared(const void* d_l, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
                            void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Scratch bytes lu_factor / cholesky_factor need (same for both). 0 on invalid arguments. */
size_t factor_workspace_bytes(int64_t n, dla_dtype dt, const dla_factor_params* p);

/*
 * 3mm: G = (A*B)*(C*D) (paper, Section "Linear Algebra Benchmarks" and the
 * 3mm_basic listing: E = A*B and F = C*D are internal temporaries, the
 * arguments are A, B, C, D and G).
 *   A ni x nk, B nk x nj, C nj x nm, D nm x nl, G ni x nl; A..D are read only,
 *   G is overwritten.  E (ni x nj) and F (nj x nl) live in the workspace
 *   (mm3_workspace_bytes), rounded to the element type between products as in
 *   the listing.  E and F are computed by one grouped launch, G by a second.
 * Any dimension equal to 0 yields an empty or all-zero G and succeeds.
 */
int mm3(const void* d_a, int64_t lda, const void* d_b, int64_t ldb, const void* d_c, int64_t ldc,
        const void* d_d, int64_t ldd, void* d_g, int64_t ldg, int64_t ni, int64_t nk, int64_t nj,
        int64_t nm, int64_t nl, dla_dtype dt, const dla_mm3_params* p, void* d_workspace,
        size_t workspace_bytes, void* hip_stream);

size_t mm3_workspace_bytes(int64_t ni, int64_t nj, int64_t nl, dla_dtype dt);

/*
 * mm3 for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result as mm3 without
 * the workspace: E and F live in a fixed scratch array that is part of the library's device image
 * (DLA_MM3_NOALLOC_MAX_BYTES per GPU, held until the process ends).  The call allocates and frees nothing
 * and enqueues the same two launches as mm3 on hip_stream.  The first call on a device looks the array's
 * device address up once (hipGetSymbolAddress).
 *   - Sizes whose E and F need more than DLA_MM3_NOALLOC_MAX_BYTES (mm3_workspace_bytes(ni, nj, nl, dt)
 *     exceeds it) are refused with DLA_ERR_TOO_LARGE before any work is enqueued; the paper's extralarge
 *     3mm (E 1600 x 1800, F 1800 x 2200 in fp64) fits.
 *   - All calls on one GPU share the one array, which keeps the previous call's E and F (nothing in it
 *     has to start at zero: every element a call reads it has written first).  Calls that overlap in
 *     time on one GPU (different streams, or several host threads) race on it: serialise them, or use
 *     mm3 with a workspace per call.
 */
#define DLA_MM3_NOALLOC_MAX_BYTES (64u << 20)
int mm3_noalloc(const void* d_a, int64_t lda, const void* d_b, int64_t ldb, const void* d_c, int64_t ldc,
                const void* d_d, int64_t ldd, void* d_g, int64_t ldg, int64_t ni, int64_t nk, int64_t nj,
                int64_t nm, int64_t nl, dla_dtype dt, const dla_mm3_params* p, void* hip_stream);

/*
 * The GEMM building block of all three kernels, exported so that a search can
 * time one schedule in isolation.
 *   op 0:  C  = A*B            A m x k, B k x n
 *   op 1:  C -= A*B            (the LU trailing update)
 *   op 2:  lower(C) -= A*B^T   A m x k, B n x k, m == n; tiles that lie strictly
 *          above the diagonal are skipped, the upper part of diagonal tiles
 *          is computed too (the Cholesky trailing update)
 *   op 3:  C -= A*B^T          A m x k, B n x k, every tile (the Cholesky look-ahead panel update)
 *   op 4:  C -= A^T*B          A k x m, B k x n (the backward pass of cholesky_solve multiplies by
 *          L^T this way); only the 32x32 (16x16 waves) and 64x64 (32x32 waves) macro-tiles, p == NULL
 *          takes the latter
 * C must not overlap A or B.
 */
int dla_gemm(int op, const void* d_a, int64_t lda, const void* d_b, int64_t ldb, void* d_c,
             int64_t ldc, int64_t m, int64_t n, int64_t k, dla_dtype dt, const dla_gemm_params* p,
             void* hip_stream);

/*
 * The default trailing update of the factorisations on its own (a step of the blocked algorithm that
 * computes the decompositions of the paper's Section "Linear Algebra Benchmarks"; the paper itself does
 * not describe a blocking), exported so that it can be timed and tested in isolation:
 *   lower == 0:  C -= L*R          L m x k, R k x m, C m x m            (LU)
 *   lower == 1:  lower(C) -= L*L^T in blocks of 128 rows: row block i is updated in columns
 *                0 .. 128*(i+1)-1, so the part of diagonal blocks above the diagonal changes too;
 *                d_r is ignored                                          (Cholesky)
 * k <= 256: up to 128 one panel of the factorisation; above that the form the factorisations use
 * for large trailing matrices, two panels at once (column blocks of 16 instead of 32, twice the
 * flops per byte of C).  All three matrices share the leading dimension ld (they are parts of one matrix in the
 * factorisations).  C must not overlap L or R.
 */
int dla_rank_update(int lower, const void* d_l, const void* d_r, void* d_c, int64_t ld, int64_t m, int64_t k,
                    dla_dtype dt, void* hip_stream);

/* 1 if the schedule is in the menu for dt (fields equal to 0 are filled with defaults first), else 0. */
int dla_gemm_params_supported(dla_dtype dt, const dla_gemm_params* p);

/*
 * Writes up to cap legal schedules to out (may be NULL when cap == 0) and
 * returns how many the menu holds: a search builds its space from this.
 */
int dla_enumerate_tiles(dla_dtype dt, dla_gemm_params* out, int cap);

/* 1 if nb is a legal block size for the factorisations (16 .. 128 step 16; 160, 192, 224, 256), else 0. */
int dla_block_size_supported(dla_dtype dt, int nb);

/*
 * Fills *out with the default schedule for a kernel (DLA_KERNEL_*) at size n:
 * out points to a dla_mm3_params for DLA_KERNEL_MM3, else to a dla_factor_params.
 */
int dla_default_params(int kernel, int64_t n, dla_dtype dt, void* out);

/*
 * Optional per-phase timing for benchmarks.  While enabled, the factorisations
 * and mm3 bracket every launch of the named phase with events on the stream
 * the kernel runs on.  dla_profile_read synchronises those events and returns
 * accumulated milliseconds and launch counts, then clears them.
 * Phases: 0 = tiled GEMM (3mm products, strip updates, caller-tiled trailing updates),
 * 1 = diagonal block, 2 = panel solves and head update, 3 = bulk trailing update (default schedule).
 * Profiling is per process, not thread safe, and perturbs the pipeline; leave
 * it off when timing whole calls.
 */
int dla_profile_enable(int on);
int dla_profile_read(int phase, double* ms_total, int64_t* launches, double* flops);

/*
 * Achievable matrix-pipe peak: runs a register-resident 16x16x4 MFMA loop of the given type on the
 * whole chip (about 2 ms, three times) and reports the fastest pass in TFLOP/s, the yardstick next
 * to the published peak when a GEMM's efficiency is quoted.  Unlike every other entry point it
 * synchronises hip_stream (it times itself with events).  d_scratch: device, 8-byte aligned, at
 * least dla_mfma_peak_scratch_bytes() bytes, overwritten.
 */
int dla_mfma_peak(dla_dtype dt, void* d_scratch, size_t scratch_bytes, void* hip_stream, double* tflops);
size_t dla_mfma_peak_scratch_bytes(void);

/*
 * Diagnostic for the look-ahead pipeline's in-kernel waits (dla_factor_params.lookahead = 1): runs one
 * diagonal-block kernel that is told to wait for a predecessor that does not exist.  After the bounded
 * poll (about 0.1 s) it gives up and reports *d_info = -1, which is what a factorisation reports where
 * kernels cannot run side by side; the kernel exits normally.  d_scratch: device, 256-byte aligned,
 * at least 8192 bytes, overwritten.  d_info: device int, must be preset by the caller (it is only
 * written on the report).
 */
int dla_handover_selftest(void* d_scratch, size_t scratch_bytes, void* hip_stream, int* d_info);

const char* dla_strerror(int code);
/*
 * After an entry point returned DLA_ERR_HIP on this host thread: which HIP error it was and in which of
 * the library's launch functions ("hipErrorX (code) in function"); "" if there was none.  The string is
 * owned by the library and overwritten by the next call on the same thread.
 */
const char* dla_last_error_detail(void);
const char* dla_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DLA_H */
