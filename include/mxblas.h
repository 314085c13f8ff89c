/*
 * mxblas — BLAS level-1 and level-2 kernels for AMD MI355X (gfx950), C ABI.
 *
 * The routines are the kernel family that the paper's two shared scheduling operators target:
 * the level-1 streaming and reduction kernels of Sec. 6.2.1 (axpy, scal, dot, asum; nrm2 is the
 * one the paper could not express and is added here from its plain definition) and the level-2
 * matrix-vector kernels of Sec. 6.2.2 (gemv in both orientations, trmv, symv, ger).  The object
 * code the paper prints fixes what each computes (gemv: Sec. 2; axpy: Fig. 4a; transposed gemv:
 * Fig. 7c); alpha/beta scaling, trans/uplo/diag, leading dimensions and increments have their
 * standard BLAS meaning (the paper's kernels "handle scaling", Sec. 6.2.2, and come in stride-1
 * and stride-any variants, Fig. 9b).
 *
 * CONVENTIONS (apply to every routine below)
 *
 *  Pointers.  Every data pointer (x, y, A, result, workspace) is a DEVICE pointer valid on the GPU
 *    that is current when the routine is called.  alpha and beta are passed by value from the
 *    host.  Reduction results (dot, asum, nrm2) are written to a device pointer, in stream order.
 *  Ownership.  The library never allocates, frees or copies device memory and never
 *    synchronises: all work is enqueued on the handle's stream and the call returns at once.
 *    Buffers must stay alive until that work has completed.  Input and output buffers must not
 *    overlap each other or the workspace (trmv's x is in place by definition).
 *  Workspace.  Routines that combine per-block partial results (dot, asum, nrm2, iamax, gemv,
 *    trmv, symv) use the handle's workspace, a caller-owned device buffer, and so does trsv, whose
 *    workgroups hand their solutions on through it; mxb_workspace_bytes gives an upper bound on
 *    what a call needs.  Partials are combined by a second kernel in a fixed order: no atomic
 *    additions, results are bitwise reproducible from run to run.
 *  Layout.  Row-major (MXB_ROW_MAJOR) is native: element (i, j) is A[i*lda + j], as in the
 *    paper's object code.  Column-major calls are remapped on the host to the row-major kernel of
 *    the transposed problem.
 *  Increments.  incx / incy may be any non-zero value unless stated; a negative increment walks
 *    the vector backwards from element (n-1)*|inc|, as in reference BLAS.
 *  Errors.  Return value 0 = success (including quick returns that launch nothing).
 *    -k  = the k-th argument after the handle is invalid (1-based); nothing was launched.
 *    MXB_ERR_*   (small positive) = handle / workspace problems; nothing was launched.
 *    MXB_ERR_HIP_BASE + hipError_t = a kernel launch failed.
 *    Argument checks touch no device state, so they also work on a host without a GPU.
 *  Threads.  A handle must not be used from two threads at once.
 */
#ifndef MXBLAS_H
#define MXBLAS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mxb_ctx* mxb_handle_t;

typedef enum { MXB_ROW_MAJOR = 101, MXB_COL_MAJOR = 102 } mxb_layout_t;
typedef enum { MXB_NO_TRANS = 111, MXB_TRANS = 112 } mxb_trans_t;
typedef enum { MXB_UPPER = 121, MXB_LOWER = 122 } mxb_uplo_t;
typedef enum { MXB_NON_UNIT = 131, MXB_UNIT = 132 } mxb_diag_t;

typedef enum {
    MXB_AXPY = 1, MXB_SCAL = 2, MXB_DOT = 3, MXB_ASUM = 4, MXB_NRM2 = 5,
    MXB_GEMV = 6, MXB_TRMV = 7, MXB_SYMV = 8, MXB_GER = 9, MXB_GEMV_BATCHED = 10, MXB_TRSV = 11
} mxb_routine_t;

#define MXB_OK 0
#define MXB_ERR_HANDLE 1          /* null or destroyed handle */
#define MXB_ERR_WORKSPACE 2       /* workspace missing or smaller than this call needs */
#define MXB_ERR_NOT_IMPLEMENTED 3
#define MXB_ERR_TIMEOUT 4         /* a kernel gave up a bounded wait (mxb_last_status) */
#define MXB_ERR_STATIC_LIMIT 5    /* mxb_sgemv_static: the call needs more scratch memory than the library's static array holds */
#define MXB_ERR_HIP_BASE 1000     /* + hipError_t of a failed launch */

/* ---- handle ------------------------------------------------------------------------------ */

/* Creates a host-side handle (stream = default stream, no workspace).  Allocates no device
 * memory and makes no GPU call.  Returns -1 if h is NULL. */
int mxb_create(mxb_handle_t* h);
int mxb_destroy(mxb_handle_t h);
/* hip_stream is a hipStream_t (borrowed); NULL selects the default stream. */
int mxb_set_stream(mxb_handle_t h, void* hip_stream);
/* dev_ptr: device buffer of `bytes` bytes, 256-byte aligned, borrowed until replaced. */
int mxb_set_workspace(mxb_handle_t h, void* dev_ptr, size_t bytes);
/* Upper bound on the workspace a call of `routine` (mxb_routine_t) with element size 4 or 8 and
 * problem size (m, n) needs; level-1 routines and trmv/symv use n only.  0 for bad arguments. */
size_t mxb_workspace_bytes(int routine, int elem_size, int64_t m, int64_t n);
/* The same bound for the launch-geometry options set on handle h (mxb_workspace_bytes assumes the
 * defaults; an option that asks for more blocks also asks for more partial results).  h == NULL
 * gives mxb_workspace_bytes.  0 for bad arguments or a bad handle. */
size_t mxb_workspace_bytes_for(mxb_handle_t h, int routine, int elem_size, int64_t m, int64_t n);

/* Launch-geometry options (per handle).  Results stay within the documented tolerance for any
 * setting and are bitwise reproducible for a fixed setting; mxb_workspace_bytes assumes the
 * defaults.  value <= 0 restores the default.  Returns -1 for an unknown option. */
typedef enum {
    MXB_OPT_L1_BLOCKS_PER_CU = 0,   /* streaming level-1 kernels: resident blocks per compute unit */
    MXB_OPT_REDUCE_BLOCKS = 1,      /* dot/asum/nrm2: maximum number of first-pass blocks (partials) */
    MXB_OPT_ROWDOT_XCHUNK = 2,      /* row-dot kernels: elements of x staged in LDS per chunk (multiple of 256) */
    MXB_OPT_ROWDOT_BLOCKS_PER_CU = 3,
    MXB_OPT_COLACC_TARGET_BLOCKS = 4, /* column-accumulate kernels: blocks to aim for when splitting rows */
    MXB_OPT_COLACC_MIN_ROWS = 5,    /* ... and the fewest rows one block may take */
    MXB_OPT_SYMV_TARGET_BLOCKS = 6, /* symv and transposed trmv (triangle sweep): grid size */
    MXB_OPT_GER_ROWS_PER_BLOCK = 7,
    MXB_OPT_SYMV_TILE_VECTORS = 8,  /* triangle sweep: 128-bit vectors per lane and row (1, 2 or 4); tile = 256 lanes x this */
    MXB_OPT_TRI_DIAG_WEIGHT = 9,    /* triangle sweep: cost of a row that crosses the diagonal, in quarters of a row that does not (1..8) */
    MXB_OPT_SYMV_SMALL_MAX = 10,    /* symv: largest n that takes the single-kernel path (every element read twice, no workspace); two thirds of it in double precision */
    MXB_OPT_TRSV_CHAIN_MIN = 11,    /* trsv: smallest n solved by the single chained kernel instead of one launch per block (default 129) */
    MXB_OPT_TRSV_SPIN_LIMIT = 12,   /* chained trsv: polls of one hand-over word before a wavefront gives up (default 2^24: tens of seconds) */
    MXB_OPT_GEMVT_SMALL_MAX = 13,   /* transposed gemv: largest matrix in bytes that takes the single-kernel path (no workspace) */
    MXB_OPT_GEMVN_SMALL_MAX = 14,   /* gemv, not transposed: largest matrix in bytes that takes the kernel for cache-resident matrices */
    MXB_OPT_COUNT = 15
} mxb_option_t;
int mxb_set_option(mxb_handle_t h, int option, int64_t value);
int64_t mxb_get_option(mxb_handle_t h, int option);

/* Waits for the handle's stream and reports what only the device knows about the last call on
 * this handle that can fail there: MXB_OK, or MXB_ERR_TIMEOUT if the last chained trsv gave up
 * a bounded wait (x is then unfinished).  The next call on the handle that uses the workspace,
 * or mxb_set_workspace, overwrites the status word and makes this MXB_OK again.  Synchronises:
 * not for use under stream capture.  Other routines cannot fail on the device. */
int mxb_last_status(mxb_handle_t h);

/* ---- level 1 (Sec. 6.2.1) ------------------------------------------------------------------ */

/* y[i] = alpha*x[i] + y[i], i < n (Fig. 4a).  Quick return: n <= 0 or alpha == 0.
 * Errors: n < 0 (-1), x NULL (-3), incx == 0 (-4), y NULL (-5), incy == 0 (-6). */
int mxb_saxpy(mxb_handle_t h, int64_t n, float alpha, const float* x, int64_t incx, float* y, int64_t incy);
int mxb_daxpy(mxb_handle_t h, int64_t n, double alpha, const double* x, int64_t incx, double* y, int64_t incy);

/* x[i] = alpha*x[i], always multiplying.  Quick return: n <= 0 or incx <= 0.
 * Errors: n < 0 (-1), x NULL (-3). */
int mxb_sscal(mxb_handle_t h, int64_t n, float alpha, float* x, int64_t incx);
int mxb_dscal(mxb_handle_t h, int64_t n, double alpha, double* x, int64_t incx);

/* *result = sum_i x[i]*y[i].  n <= 0 writes 0.  s: products and per-thread sums in fp32, partial
 * sums combined in fp64; d: fp64 throughout.
 * Errors: n < 0 (-1), x NULL (-2), incx == 0 (-3), y NULL (-4), incy == 0 (-5), result NULL (-6). */
int mxb_sdot(mxb_handle_t h, int64_t n, const float* x, int64_t incx, const float* y, int64_t incy, float* result);
int mxb_ddot(mxb_handle_t h, int64_t n, const double* x, int64_t incx, const double* y, int64_t incy, double* result);

/* *result = sum_i |x[i]|.  n <= 0 or incx <= 0 writes 0.
 * Errors: n < 0 (-1), x NULL (-2), result NULL (-4). */
int mxb_sasum(mxb_handle_t h, int64_t n, const float* x, int64_t incx, float* result);
int mxb_dasum(mxb_handle_t h, int64_t n, const double* x, int64_t incx, double* result);

/* *result = sqrt(sum_i x[i]^2).  n <= 0 or incx <= 0 writes 0.  snrm2 squares and sums in fp64,
 * so it cannot overflow; dnrm2 sums scaled squares in three exponent ranges (Blue's method), so
 * it neither overflows nor underflows for finite inputs.
 * Errors: n < 0 (-1), x NULL (-2), result NULL (-4). */
int mxb_snrm2(mxb_handle_t h, int64_t n, const float* x, int64_t incx, float* result);
int mxb_dnrm2(mxb_handle_t h, int64_t n, const double* x, int64_t incx, double* result);

/* ---- rest of the paper's level-1 set (Sec. 6.2.1: copy, swap, rot, rotm, dsdot) and iamax -------
 * Common errors of the two-vector routines: n < 0 (-1), x NULL (-2), incx == 0 (-3), y NULL (-4),
 * incy == 0 (-5).  n == 0 launches nothing. */

/* y[i] = x[i]. */
int mxb_scopy(mxb_handle_t h, int64_t n, const float* x, int64_t incx, float* y, int64_t incy);
int mxb_dcopy(mxb_handle_t h, int64_t n, const double* x, int64_t incx, double* y, int64_t incy);
/* x[i] <-> y[i]. */
int mxb_sswap(mxb_handle_t h, int64_t n, float* x, int64_t incx, float* y, int64_t incy);
int mxb_dswap(mxb_handle_t h, int64_t n, double* x, int64_t incx, double* y, int64_t incy);
/* (x[i], y[i]) := (c*x[i] + s*y[i], c*y[i] - s*x[i]). */
int mxb_srot(mxb_handle_t h, int64_t n, float* x, int64_t incx, float* y, int64_t incy, float c, float s);
int mxb_drot(mxb_handle_t h, int64_t n, double* x, int64_t incx, double* y, int64_t incy, double c, double s);
/* (x[i], y[i]) := H (x[i], y[i]).  param is a HOST pointer to 5 values {flag, h11, h21, h12, h22}:
 * flag -1: H = [h11 h12; h21 h22]; 0: [1 h12; h21 1]; 1: [h11 1; -1 h22]; -2: identity (no launch).
 * Extra error: param NULL (-6). */
int mxb_srotm(mxb_handle_t h, int64_t n, float* x, int64_t incx, float* y, int64_t incy, const float* param);
int mxb_drotm(mxb_handle_t h, int64_t n, double* x, int64_t incx, double* y, int64_t incy, const double* param);
/* *result (double, device) = sum_i x[i]*y[i] with fp32 inputs, exact fp64 products and fp64 sums.
 * Errors as mxb_sdot. */
int mxb_dsdot(mxb_handle_t h, int64_t n, const float* x, int64_t incx, const float* y, int64_t incy, double* result);
/* *result (int64, device) = 0-based index of the first element of largest |x[i]|, as found by the
 * sequential scan that only replaces its candidate on a strictly greater magnitude (so NaN is
 * never chosen unless it is x[0]).  n <= 0 or incx <= 0 writes 0.  Uses the workspace.
 * Errors: n < 0 (-1), x NULL (-2), result NULL (-4). */
int mxb_isamax(mxb_handle_t h, int64_t n, const float* x, int64_t incx, int64_t* result);
int mxb_idamax(mxb_handle_t h, int64_t n, const double* x, int64_t incx, int64_t* result);

/* ---- level 2 (Sec. 6.2.2) ------------------------------------------------------------------ */

/* y = alpha*op(A)*x + beta*y, A m x n (Sec. 2: y[i] += A[i,j]*x[j]; Fig. 7c for op = transpose:
 * y[j] += x[i]*A[i,j]).  x has n (no-trans) or m (trans) elements, y the other count.
 * beta == 0: y is overwritten and never read.  alpha == 0: A and x are never read.
 * lda >= max(1, n) row-major, >= max(1, m) column-major.
 * Quick return: m == 0, n == 0, or (alpha == 0 and beta == 1).
 * Errors: layout (-1), trans (-2), m < 0 (-3), n < 0 (-4), A NULL (-6), lda (-7), x NULL (-8),
 *         incx == 0 (-9), y NULL (-11), incy == 0 (-12). */
int mxb_sgemv(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, float alpha,
              const float* A, int64_t lda, const float* x, int64_t incx, float beta, float* y, int64_t incy);
int mxb_dgemv(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, double alpha,
              const double* A, int64_t lda, const double* x, int64_t incx, double beta, double* y, int64_t incy);

/* mxb_sgemv for callers that cannot allocate device memory: code that runs under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bitwise the same result as mxb_sgemv, but the partial vectors that mxb_sgemv keeps in the
 * handle's workspace live in a static device array of MXB_STATIC_SCRATCH_BYTES inside the library
 * (every GPU the library runs on holds one copy until the process ends), so no workspace has to
 * be set.  The handle's workspace, if any, is neither used nor changed.  Neither this call nor
 * anything it calls allocates or frees memory; the first call on a device looks the array's
 * address up once.
 * Limit: a call whose partial vectors need more than MXB_STATIC_SCRATCH_BYTES returns
 * MXB_ERR_STATIC_LIMIT and launches nothing.  Products that are not transposed (row-major) need at
 * most 64 KiB.  A transposed product of a row-major matrix needs one partial vector per row group,
 * about 3 MiB in all with the default options whatever the shape (16384 x 16384: 48 vectors of
 * 16384 floats), and more only for rows of several hundred thousand columns, where even two row
 * groups exceed the array (512 x 782336: 6 MiB, rejected), or with raised launch-geometry options.
 * mxb_workspace_bytes(MXB_GEMV, 4, m, n) <= MXB_STATIC_SCRATCH_BYTES is sufficient for any
 * orientation.
 * All calls on one GPU share the one array: two calls that may run at the same time on one GPU
 * (different streams, different handles, different threads) race on it; calls on one stream are
 * ordered and safe.  The array keeps the last call's partial vectors; every call overwrites what
 * it reads, so nothing is cleared.
 * Errors: as mxb_sgemv, plus MXB_ERR_STATIC_LIMIT. */
#define MXB_STATIC_SCRATCH_BYTES (4u << 20)
int mxb_sgemv_static(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, float alpha,
                     const float* A, int64_t lda, const float* x, int64_t incx, float beta, float* y, int64_t incy);

/* `batch` independent gemv problems of one shape in one call (Sec. 6.2.2 gemv; for matrices so
 * small that a single product cannot fill the device): for b in [0, batch)
 *     y_b = alpha*op(A_b)*x_b + beta*y_b,   A_b = A + b*strideA, x_b = x + b*stridex, y_b = y + b*stridey
 * with the strides in elements.  Every other argument means what it means for gemv and holds for
 * all problems.  strideA == 0 or stridex == 0 shares that operand among the problems; the y_b must
 * not overlap each other (stridey == 0 is rejected for batch > 1; other overlaps are undefined).
 * All pointers are device pointers; the caller owns them.  Workspace: the bound of
 * mxb_workspace_bytes(MXB_GEMV_BATCHED, ..) holds for any batch.
 * Quick return: m == 0, n == 0, batch == 0, or (alpha == 0 and beta == 1).
 * Errors: layout (-1), trans (-2), m < 0 (-3), n < 0 (-4), A NULL (-6), lda (-7), strideA < 0 (-8),
 *         x NULL (-9), incx == 0 (-10), stridex < 0 (-11), y NULL (-13), incy == 0 (-14),
 *         stridey (-15), batch < 0 (-16). */
int mxb_sgemv_batched(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, float alpha,
                      const float* A, int64_t lda, int64_t strideA, const float* x, int64_t incx, int64_t stridex,
                      float beta, float* y, int64_t incy, int64_t stridey, int64_t batch);
int mxb_dgemv_batched(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, double alpha,
                      const double* A, int64_t lda, int64_t strideA, const double* x, int64_t incx, int64_t stridex,
                      double beta, double* y, int64_t incy, int64_t stridey, int64_t batch);

/* x := op(T)*x, T the uplo triangle of the n x n matrix A (Sec. 6.2.2, triangular matrices).
 * Elements outside the triangle are never used; with MXB_UNIT the diagonal is taken as 1 and
 * never used.  The product is formed from the x passed in (copied to the workspace first).
 * Quick return: n == 0.
 * Errors: layout (-1), uplo (-2), trans (-3), diag (-4), n < 0 (-5), A NULL (-6), lda < max(1,n)
 *         (-7), x NULL (-8), incx == 0 (-9). */
int mxb_strmv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, mxb_trans_t trans, mxb_diag_t diag,
              int64_t n, const float* A, int64_t lda, float* x, int64_t incx);
int mxb_dtrmv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, mxb_trans_t trans, mxb_diag_t diag,
              int64_t n, const double* A, int64_t lda, double* x, int64_t incx);

/* Solves op(T)*z = x for z, which overwrites x: T is the uplo triangle of the n x n matrix A
 * (Sec. 6.2.2, trsv); with MXB_UNIT the diagonal is taken as 1 and never used.  Elements outside
 * the triangle are never used.  No test for singularity.  Blocked substitution: the diagonal
 * elements enter as reciprocals (one extra rounding per unknown).  Below MXB_OPT_TRSV_CHAIN_MIN
 * unknowns: one launch per block of 512 (fp32) or 256 (fp64) unknowns, with the workspace used when
 * the product is transposed (as gemv does).  From there on: one kernel whose workgroups solve 256
 * unknowns each, in order, and hand the solved values on through the workspace (16 bytes per
 * unknown at most, cleared by the call; MXB_ERR_WORKSPACE if it is smaller).  A workgroup waits
 * for solved values a bounded number of polls only (MXB_OPT_TRSV_SPIN_LIMIT); the bound (tens of
 * seconds) is reached only if the device stops scheduling the workgroup that owns them; x is
 * then left unfinished and mxb_last_status reports MXB_ERR_TIMEOUT.
 * mxb_workspace_bytes(MXB_TRSV, elem_size, 0, n) covers both paths.
 * Quick return: n == 0.
 * Errors: as mxb_strmv. */
int mxb_strsv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, mxb_trans_t trans, mxb_diag_t diag,
              int64_t n, const float* A, int64_t lda, float* x, int64_t incx);
int mxb_dtrsv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, mxb_trans_t trans, mxb_diag_t diag,
              int64_t n, const double* A, int64_t lda, double* x, int64_t incx);

/* y = alpha*S*x + beta*y, S symmetric n x n, only the uplo triangle of A is used (Sec. 6.2.2).
 * beta == 0 / alpha == 0 as for gemv.  Quick return: n == 0 or (alpha == 0 and beta == 1).
 * Errors: layout (-1), uplo (-2), n < 0 (-3), A NULL (-5), lda < max(1,n) (-6), x NULL (-7),
 *         incx == 0 (-8), y NULL (-10), incy == 0 (-11). */
int mxb_ssymv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, float alpha, const float* A,
              int64_t lda, const float* x, int64_t incx, float beta, float* y, int64_t incy);
int mxb_dsymv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, double alpha, const double* A,
              int64_t lda, const double* x, int64_t incx, double beta, double* y, int64_t incy);

/* A[i,j] += alpha*x[i]*y[j], A m x n, x has m elements, y has n (Sec. 6.2.2).
 * Quick return: m == 0, n == 0 or alpha == 0.
 * Errors: layout (-1), m < 0 (-2), n < 0 (-3), x NULL (-5), incx == 0 (-6), y NULL (-7),
 *         incy == 0 (-8), A NULL (-9), lda (-10). */
int mxb_sger(mxb_handle_t h, mxb_layout_t layout, int64_t m, int64_t n, float alpha, const float* x, int64_t incx,
             const float* y, int64_t incy, float* A, int64_t lda);
int mxb_dger(mxb_handle_t h, mxb_layout_t layout, int64_t m, int64_t n, double alpha, const double* x, int64_t incx,
             const double* y, int64_t incy, double* A, int64_t lda);

/* A[i,j] += alpha*x[i]*x[j] for (i, j) in the uplo triangle of the n x n matrix A (Sec. 6.2.2,
 * syr).  Nothing outside the triangle is read or written.  Quick return: n == 0 or alpha == 0.
 * Errors: layout (-1), uplo (-2), n < 0 (-3), x NULL (-5), incx == 0 (-6), A NULL (-7),
 *         lda < max(1,n) (-8). */
int mxb_ssyr(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, float alpha, const float* x, int64_t incx,
             float* A, int64_t lda);
int mxb_dsyr(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, double alpha, const double* x, int64_t incx,
             double* A, int64_t lda);

/* A[i,j] += alpha*x[i]*y[j] + alpha*y[i]*x[j] for (i, j) in the uplo triangle (Sec. 6.2.2, syr2).
 * Quick return: n == 0 or alpha == 0.
 * Errors: layout (-1), uplo (-2), n < 0 (-3), x NULL (-5), incx == 0 (-6), y NULL (-7),
 *         incy == 0 (-8), A NULL (-9), lda < max(1,n) (-10). */
int mxb_ssyr2(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, float alpha, const float* x, int64_t incx,
              const float* y, int64_t incy, float* A, int64_t lda);
int mxb_dsyr2(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, double alpha, const double* x, int64_t incx,
              const double* y, int64_t incy, double* A, int64_t lda);

/* ---- bandwidth probes (measurement aids, not BLAS) ----------------------------------------- */

/* dst[0..bytes) = src[0..bytes) with the same 128-bit streaming loads/stores the kernels use.
 * bytes must be a multiple of 16 and both pointers 16-byte aligned (else -1). */
int mxb_probe_copy(mxb_handle_t h, size_t bytes, const void* src, void* dst);
/* Reads src[0..bytes) and writes one 8-byte checksum per block to the workspace: what a pure
 * read stream reaches on this device. */
int mxb_probe_read(mxb_handle_t h, size_t bytes, const void* src);

#ifdef __cplusplus
}
#endif
#endif /* MXBLAS_H */
