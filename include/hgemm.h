/*
 * hgemm.h -- C ABI of the MI355X (gfx950) half-precision GEMM library.
 *
 * The operation (paper Section 2.1, "HGEMM"): C = alpha*A*B + beta*C with
 * alpha = 1, beta = 0, i.e. C = A*B, where A is M x K, B is K x N, C is M x N,
 * all stored as IEEE binary16.  Products are accumulated in fp32 (one of the
 * two accumulator choices Section 1 names as valid for fp16 inputs) and each
 * result is rounded once, to nearest even, to fp16.
 *
 * Layouts (Section 2.2.2): "NN" = A, B, C all row-major; "TN" = B stored
 * column-major (an N x K row-major array).  A and C are always row-major.
 *
 * One plan per (M,N,K,layout): the paper's premise (Abstract, Section 5) is
 * that every shape wants its own kernel configuration; hgemm_plan() looks the
 * shape up in a table of measured choices (one table per layout of B; a shape
 * tuned only with row-major B uses that row for column-major B too) and falls
 * back to a fitted cost model.
 *
 * Threading: functions are thread-compatible (no global mutable state apart
 * from a read-only table and two per-device caches behind mutexes: whether a
 * device is a gfx950, and the address of hgemm_run_static's scratch array); a
 * single plan must not be run on two streams at once because split-K,
 * stream-K and padded plans own a workspace.
 * The library never prints, never throws, never synchronises the device, and
 * launches only on the stream it is given (Section 2.4.1 forbids a kernel
 * under test from using extra streams).
 */
#ifndef HGEMM_H
#define HGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hgemm_plan_s* hgemm_plan_t;      /* opaque; owned by the library */

typedef enum {
    HGEMM_OK              = 0,
    HGEMM_ERR_INVALID_ARG = 1,   /* null pointer, negative size, bad enum, bad spec string */
    HGEMM_ERR_UNSUPPORTED = 2,   /* layout / leading dimension / alignment not implemented */
    HGEMM_ERR_ALLOC       = 3,   /* workspace allocation failed                            */
    HGEMM_ERR_LAUNCH      = 4,   /* the HIP runtime reported a launch error                */
    HGEMM_ERR_ARCH        = 5,   /* current device is not gfx950                           */
    HGEMM_ERR_WORKSPACE   = 6    /* hgemm_run_static: the plan needs more scratch than the
                                    static buffer holds                                    */
} hgemm_status_t;

typedef enum { HGEMM_ROW_MAJOR = 0, HGEMM_COL_MAJOR = 1 } hgemm_layout_t;

/* Storage of the three matrices.  ld* are leading dimensions in ELEMENTS;
 * 0 means packed (lda = K, ldb = N for row-major B or K for column-major B,
 * ldc = N).  a and c must be HGEMM_ROW_MAJOR.                               */
typedef struct {
    hgemm_layout_t a, b, c;
    int64_t lda, ldb, ldc;
} hgemm_layouts_t;

/*
 * hgemm_plan -- choose a kernel specialisation for one shape (Section 5: tile
 * sizes BM/BN/BK, stage count, block swizzle and the rest are picked per
 * (M,N,K)).  Host only: no kernel is launched.
 *   out      receives the plan (host pointer, written on HGEMM_OK only)
 *   M,N,K    >= 0.  M, N or K equal to 0 is valid (K = 0 gives C = 0).
 *   layouts  host pointer; NULL means NN, packed
 * Allocates the plan's device workspace (split-K partial sums, stream-K
 * partial tiles, padded copies of unaligned operands) on the CURRENT device,
 * if the choice needs one.
 * Size: the matrix-core kernels address an operand with 32-bit byte offsets,
 * i.e. up to 2 GiB of it.  A problem with a larger A, B or C (dimensions and
 * leading dimensions multiples of 8) is planned as a grid of blocks -- row
 * blocks of A and C by column panels of B and C, each a plan of its own run
 * on offset pointers, one after the other on the stream; a row-major B of
 * that size is first copied, transposed, into the workspace (2*K*N bytes
 * more), because only a K-contiguous B can be cut into panels of less than
 * 2 GiB.  hgemm_plan_describe() then starts with "blocks,rows=R,cols=C".
 * Only hgemm_plan() does this: an explicit spec returns UNSUPPORTED for
 * such a problem, and hgemm_run_static() runs it on the generic kernel.
 * Errors: INVALID_ARG, UNSUPPORTED, ALLOC, ARCH.
 */
hgemm_status_t hgemm_plan(hgemm_plan_t* out, int64_t M, int64_t N, int64_t K,
                          const hgemm_layouts_t* layouts);

/*
 * hgemm_plan_override -- as hgemm_plan, but with the specialisation given by
 * `spec` instead of the dispatch table; used by the autotuner and by tests
 * that must cover every kernel.  `spec` is a host string of the form
 *   "<family>[,key=value]..."    e.g.  "mfma,bm=256,bn=256,bk=64,st=2,sk=1"
 * Families and keys are listed by hgemm_spec_help().  One key changes the
 * arithmetic rather than the schedule: "ac=16" asks for a 16-bit accumulator
 * (Section 1: fp16 and fp32 accumulators are both valid for fp16 inputs;
 * Section 2.3.2's exact-match test is built for the former): the running
 * sums are rounded to fp16 after every 16 products.  hgemm_plan() never
 * chooses it.  A spec that cannot run
 * the shape as it lies in memory (alignment, tile larger than the limits)
 * returns UNSUPPORTED: an explicit spec never pads.
 */
hgemm_status_t hgemm_plan_override(hgemm_plan_t* out, int64_t M, int64_t N, int64_t K,
                                   const hgemm_layouts_t* layouts, const char* spec);

/*
 * hgemm_run -- enqueue C = A*B on `hip_stream` (Section 2.1; the call shape
 * kernel(a, b, out) of Section 2.4.1's timing listing).
 *   A, B, C     DEVICE pointers to fp16, owned by the caller, non-overlapping.
 *               The matrix-core kernels need 16-byte aligned bases and K, N
 *               (and the leading dimensions) multiples of 8.  When K, N or a
 *               leading dimension is not, hgemm_plan() arranges zero-padded
 *               packed copies of A, B and C in the plan's workspace (Section
 *               5.2's zero padding; two copy kernels before and one after the
 *               GEMM, on the same stream), except for problems below 2^20
 *               multiply-adds, which take a generic one-thread-per-element
 *               kernel, as do calls whose base pointers are not 16-byte
 *               aligned.  C is write-only: every element is overwritten
 *               (beta = 0), earlier contents never leak, and nothing outside
 *               the M x N elements of C is written.
 *   hip_stream  a hipStream_t passed as void*; NULL = the default stream.
 * Asynchronous; allocates nothing; all kernels (main, split-K reduction,
 * stream-K fix-up, the optional transposing copy of B) go to hip_stream in
 * order.
 * Errors: INVALID_ARG (null plan / null pointer with a non-empty problem),
 * LAUNCH.
 */
hgemm_status_t hgemm_run(hgemm_plan_t plan, const void* A, const void* B, void* C,
                         void* hip_stream);

/*
 * hgemm_run_many -- enqueue `count` calls of one plan back to back on
 * `hip_stream` (Section 2.4.2's offline mode: the same kernel executed
 * consecutively, without pauses).  Call i works on operand set j = (first + i)
 * % sets, C[j] = A[j] * B[j]; the result is that of `count` calls of hgemm_run
 * in a loop.  The
 * loop runs inside the library so that a caller in an interpreted language
 * pays its per-call overhead once per batch: kernels of 2-3 us are otherwise
 * enqueued more slowly than the GPU executes them.
 *   count       number of calls, >= 0
 *   sets        number of operand sets, >= 1
 *   first       set of the first call, 0 <= first < sets (a caller that cycles
 *               through sets larger than the caches continues where its last
 *               batch stopped)
 *   A, B, C     HOST arrays of `sets` DEVICE pointers each (read during the
 *               call only); the operands they point to are as in hgemm_run
 *   hip_stream  as hgemm_run
 * Errors: as hgemm_run; stops at the first call that fails (calls already
 * enqueued stay enqueued).
 */
hgemm_status_t hgemm_run_many(hgemm_plan_t plan, int64_t count, int64_t sets, int64_t first,
                              const void* const* A, const void* const* B, void* const* C,
                              void* hip_stream);

/*
 * hgemm_run_static -- plan and enqueue C = A*B in one call that allocates
 * nothing, for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same operation,
 * argument meaning and kernels as hgemm_plan() + hgemm_run(); the difference
 * is where the workspace lives.  Split-K planes, stream-K partial tiles and
 * the padded copies of unaligned operands go to a static device array of
 * HGEMM_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until
 * the process ends) instead of a hipMalloc'ed buffer, and the plan itself
 * lives on the call's stack.  A problem whose chosen specialisation needs more
 * scratch than that returns HGEMM_ERR_WORKSPACE and launches nothing; problems
 * that need no workspace are never refused.  The kernels overwrite every
 * scratch element they later read, so nothing has to be cleared between calls.
 * All calls on one GPU share that GPU's array: calls whose kernels may overlap
 * in time (different streams, no dependency between them) race on it, and so
 * does a call overlapping nothing but itself replayed concurrently from two
 * graphs.  Calls on one stream are safe.
 *   M,N,K,layouts   as hgemm_plan (host values); A,B,C,hip_stream as hgemm_run
 * Errors: INVALID_ARG, UNSUPPORTED, ARCH, WORKSPACE, LAUNCH.
 */
#define HGEMM_STATIC_SCRATCH_BYTES (64u << 20)
hgemm_status_t hgemm_run_static(int64_t M, int64_t N, int64_t K, const hgemm_layouts_t* layouts,
                                const void* A, const void* B, void* C, void* hip_stream);

/* hgemm_destroy -- free the plan and its workspace.  NULL is accepted.
 * (Housekeeping of this interface; the paper has no passage to cite for it,
 * nor for hgemm_status_string and hgemm_plan_describe below.)               */
hgemm_status_t hgemm_destroy(hgemm_plan_t plan);

/* ---- helpers (not on the hot path) --------------------------------------- */

/* Static, NUL-terminated description of a status code.                      */
const char* hgemm_status_string(hgemm_status_t status);

/* Writes the chosen specialisation as a spec string (same grammar as
 * hgemm_plan_override accepts) into buf[0..n), always NUL-terminated.
 * Returns INVALID_ARG when buf is NULL, n is 0, or the text does not fit.   */
hgemm_status_t hgemm_plan_describe(hgemm_plan_t plan, char* buf, size_t n);

/* Device workspace bytes owned by the plan (0 for single-pass kernels).     */
size_t hgemm_plan_workspace_bytes(hgemm_plan_t plan);

/* Number of workgroups of the plan's main kernel and its LDS bytes per
 * workgroup; for reports.  Either out pointer may be NULL.                  */
hgemm_status_t hgemm_plan_launch_info(hgemm_plan_t plan, int64_t* workgroups,
                                      int64_t* lds_bytes, int64_t* threads);

/* Static text listing the kernel families and the keys a spec may carry.    */
const char* hgemm_spec_help(void);

/* Candidate specs worth timing for a shape (the autotuner's search space,
 * seeded by the trends of Section 6: tiles grow with M and N, stages with K).
 * Fills buf with specs separated by '\n'; returns INVALID_ARG if it does not
 * fit.                                                                      */
hgemm_status_t hgemm_candidates(int64_t M, int64_t N, int64_t K,
                                const hgemm_layouts_t* layouts, char* buf, size_t n);

/* What hgemm_plan() would choose for a problem, and why, without a device
 * (host only; nothing is allocated or launched): buf receives one of
 *   "table: SPEC"      the row of the layout's dispatch table (Section 5: one
 *                      configuration per (M,N,K), here from timed runs)
 *   "neighbour: SPEC"  a large problem the table does not hold: the kernel
 *                      tuned for the nearest shape it does hold
 *   "model: SPEC"      the fitted cost model's pick;  "rules: SPEC" its last
 *                      resort
 *   "blocks,rows=R,cols=C[,bt=1]"   operands of 2 GiB and more
 *   "generic"          unaligned and too small to pad;  "empty"  M, N or K = 0
 * with ",pad=1" appended when the kernel would run on zero-padded copies.
 * hgemm_plan() then still has to set the choice up on the device; where that
 * fails (a kernel this build lacks, no memory) it falls back as documented
 * there.  Errors: INVALID_ARG (also when buf is too small), UNSUPPORTED.    */
hgemm_status_t hgemm_plan_choice(int64_t M, int64_t N, int64_t K,
                                 const hgemm_layouts_t* layouts, char* buf, size_t n);

/* The planner's cost model: predicted microseconds of one call of `spec` (an "mfma" spec without
 * tb/sm) on an M x N x K problem.  hgemm_plan() picks the compiled configuration and split factor
 * with the smallest prediction when its measured table has no row for the shape (Section 6 reads
 * such trends -- tile size against M and N, stages against K -- off the paper's winners; here they
 * are a fitted model of one launch).  Host only.  Errors: INVALID_ARG, UNSUPPORTED.            */
hgemm_status_t hgemm_predict_us(int64_t M, int64_t N, int64_t K, const char* spec, double* us);

/* Tile-count arithmetic of the zero-padding technique (Section 5.2): number
 * of tiles along a dimension of size `dim` with tile size `tile`, and the
 * padded size tiles*tile.  Out-of-range rows/columns are read as zeros and
 * never stored, so no tile size needs to divide the dimension.              */
int64_t hgemm_tiles(int64_t dim, int64_t tile);
int64_t hgemm_padded(int64_t dim, int64_t tile);

/* Tile -> workgroup mapping (Section 5.3 "block swizzle", Section 6.3),
 * re-thought for 8 XCDs with private L2 caches: maps the linear workgroup id
 * the hardware dispatches round-robin over XCDs to a (tile_m, tile_n) pair so
 * that the workgroups resident on one XCD cover a compact block of tiles.
 * Host-side mirror of the device function, exported for tests.
 * Returns tile_m * tiles_n + tile_n, or -1 for bad arguments.               */
int64_t hgemm_tile_of_workgroup(int64_t wg, int64_t tiles_m, int64_t tiles_n,
                                int64_t swizzle);

/* Calibration kernels for the roofline (not part of any GEMM): run `iters`
 * dependent-free MFMA instructions per wave on every CU / stream `bytes`
 * bytes from `src` (device pointer) and return the elapsed milliseconds
 * measured with events on `hip_stream`.  These two calls synchronise.       */
hgemm_status_t hgemm_calibrate_mfma(int64_t iters, void* hip_stream, double* ms, double* flop);
hgemm_status_t hgemm_calibrate_hbm_read(const void* src, size_t bytes, void* hip_stream, double* ms);

#ifdef __cplusplus
}
#endif
#endif /* HGEMM_H */
