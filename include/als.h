/*
 * libals — implicit Alternating Least Squares (iALS) half-epoch solve on one AMD MI355X (gfx950).
 *
 * Plain C ABI.  Every pointer marked "device" is HIP device memory on the
 * context's GPU; "host" pointers are ordinary host memory.  The caller owns
 * every buffer it passes; the library owns only the workspace held by an
 * als_ctx and never frees or reallocates caller memory.  No C++ exception
 * crosses this boundary: every entry point returns an als_status.
 *
 * Notation follows the paper (ALX, Section 3): a sparse label matrix Y
 * (m rows "users" x n columns "items"), embedding tables W [m x d] and
 * H [n x d], prediction <w_u, h_i>, unobserved weight alpha, L2 weight lambda.
 * The objective is Eq. 3; one half-epoch replaces every row of one table by
 * the exact minimiser of Eq. 3 with the other table held fixed (Eq. 4,
 * Algorithm 1 lines 2-10).
 */
#ifndef ALS_H
#define ALS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ALS_OK = 0,
    ALS_EINVAL = 1,  /* null pointer, negative size, bad parameter value            */
    ALS_ESHAPE = 2,  /* shapes of the arguments do not fit each other               */
    ALS_EDTYPE = 3,  /* unsupported element type or d, or tables of different types */
    ALS_EALIAS = 4,  /* output table overlaps an input table                        */
    ALS_ENOTSPD = 5, /* lambda <= 0, or a non-positive pivot met on the device      */
    ALS_ENOMEM = 6,  /* workspace allocation failed                                 */
    ALS_EHIP = 7     /* a HIP runtime call failed (see als_last_error)              */
} als_status;

typedef enum { ALS_F32 = 0, ALS_BF16 = 1 } als_dtype;

/* Which formulation als_solve_rows uses for a row with k stored entries.
 *   ALS_PATH_AUTO   : rows with 0 < k <= dual_max_k use the k x k dual system,
 *                     all others the d x d normal equations.
 *   ALS_PATH_PRIMAL : every row forms and solves the d x d normal equations of
 *                     Eq. 4 (Algorithm 1 lines 4-10 literally).
 *   ALS_PATH_DUAL   : as AUTO (kept distinct so callers can state intent).
 * Both formulations reach the same minimiser of Eq. 3 (the algebra is in the header
 * comment of csrc/dual_prepare.hip).  The dual form is available for k <= min(d, 64),
 * and for k <= 128 when d = 128. */
typedef enum { ALS_PATH_AUTO = 0, ALS_PATH_PRIMAL = 1, ALS_PATH_DUAL = 2 } als_path;

/* Sparse label matrix in CSR form (Section 3: the training set S as a matrix Y).
 * Entries of a row may be in any order; every stored entry is one term of the
 * sums in Eq. 4 (duplicates are not merged). */
typedef struct {
    int64_t rows, cols, nnz;
    const int64_t *indptr; /* device [rows+1], non-decreasing, indptr[0]=0, indptr[rows]=nnz */
    const int32_t *indices; /* device [nnz], 0 <= id < cols                                   */
    const float *values;    /* device [nnz] labels y, or NULL meaning y = 1 for every entry    */
} als_csr;

/* Embedding table, row-major: element (r, c) at data[r*ld + c], 0 <= c < d.
 * Supported d: 16, 32, 64, 128.  ld is in elements and must be >= d and keep
 * rows 16-byte aligned (ld*sizeof(element) % 16 == 0; data 16-byte aligned). */
typedef struct {
    void *data; /* device */
    int64_t rows;
    int32_t d;
    int64_t ld;
    als_dtype dtype; /* ALS_F32, or ALS_BF16 (Section 4.4: bf16 storage, fp32 arithmetic) */
} als_table;

/* How a row's linear system is solved (Section 4.5 compares such solvers and settles on conjugate gradients):
 *   ALS_SOLVER_DIRECT  : Cholesky-type factorisation (exact up to rounding), of the d x d system of rows taking
 *                        the primal form and of the k x k system of rows taking the dual form.
 *   ALS_SOLVER_CG      : conjugate gradients on the assembled system, stopped when |residual| <= cg_tol * |b|
 *                        (or <= 1e-15, below which fp32 squares of it carry no information) or after
 *                        cg_max_iters iterations.  Rows taking the primal form start from their
 *                        current content in X (warm start; X must hold finite numbers); rows taking the dual
 *                        form solve their k x k system from zero (available for d >= 64; for smaller d every
 *                        row takes the primal form under this solver).
 *   ALS_SOLVER_CG_FREE : conjugate gradients on the d x d system without assembling it: a product with the
 *                        row's matrix is taken as (alpha G + lambda I) p + V_I^T (V_I p), the first term for
 *                        sixteen rows at a time as one matrix product.  Used for the rows that ALS_PATH_AUTO /
 *                        ALS_PATH_DUAL would solve in the dual form (0 < k <= dual_max_k), warm-started from X;
 *                        longer rows, and every row under ALS_PATH_PRIMAL, are solved as with ALS_SOLVER_CG. */
typedef enum { ALS_SOLVER_DIRECT = 0, ALS_SOLVER_CG = 1, ALS_SOLVER_CG_FREE = 2 } als_solver;

typedef struct {
    float alpha;        /* weight of the all-pairs term of Eq. 3, >= 0                         */
    float lambda;       /* L2 weight of Eq. 3, > 0 (keeps every system positive definite)      */
    int32_t path;       /* als_path                                                             */
    int32_t dual_max_k; /* 0 = library default (the largest supported); largest k solved in the dual
                           form, clipped to what the table's d supports                          */
    int32_t split_nnz;  /* 0 = library default; rows longer than this are cut into segments whose
                           partial statistics are summed (Section 4.3's row splitting)           */
    int32_t solver;       /* als_solver                                                          */
    int32_t cg_max_iters; /* 0 = library default (2*d)                                           */
    float cg_tol;         /* 0 = library default (1e-6); relative residual at which CG stops     */
} als_params;

typedef struct als_ctx als_ctx;

/* Create / destroy a context bound to one GPU.  als_create sets that device
 * current for the calling thread.  Workspace grows on demand and is released
 * by als_destroy.  Calls on one context must not overlap. */
als_status als_create(als_ctx **ctx, int device);
als_status als_destroy(als_ctx *ctx);

/* G = V^T V, the Gramian of a table (Section 3 after Eq. 4; Algorithm 1 line 2).
 * G: device fp32 [d*d], row-major, both triangles written, symmetric to the bit.
 * bf16 entries are used exactly (their products are exact in fp32).  For d >= 64 the products run on the bf16
 * matrix cores; fp32 entries are cut exactly into three bf16 parts there and a product keeps every term down to
 * the rounding of an fp32 product.  Sums are fp32 - inside the matrix core over short chains only (its running
 * sum is not rounded to nearest), on the vector units or in fp64 across steps and blocks of rows - in a fixed
 * order.  Asynchronous on `stream` (a hipStream_t, NULL = default). */
als_status als_gramian(als_ctx *ctx, const als_table *V, float *G, void *stream);

/* als_gramian for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  No context; calls no hipMalloc, hipFree or any other allocating
 * routine.  The per-workgroup partial sums live in a static device array of 10 MiB that every GPU the library
 * runs on holds until the process ends; it fits tables of at most ALS_GRAMIAN_STATIC_MAX_ROWS rows, larger
 * ones are refused with ALS_ESHAPE.  `device` must be the calling thread's current device.  Same kernels,
 * same summation order and therefore the same bits as als_gramian.  The address of the array is looked up
 * once per device, by als_create or by the first call (so make one of the two before capturing a graph).
 * All calls on one GPU share the array: calls that overlap in time on one GPU (different streams or
 * threads) race and give wrong sums; calls on one stream are ordered and safe.  On failure
 * als_static_last_error() holds the reason (per thread). */
#define ALS_GRAMIAN_STATIC_MAX_ROWS 262144
als_status als_gramian_static(int device, const als_table *V, float *G, void *stream);
const char *als_static_last_error(void);

/* Row update of Eq. 4 (Algorithm 1 lines 3-10) for rows row_begin <= u < row_end of Y:
 *     X[u] = ( sum_{i in Y[u]} v_i (x) v_i + alpha*G + lambda*I )^{-1} sum_{i in Y[u]} y_ui v_i
 * with v_i the rows of the fixed table V (V->rows == Y->cols) and G = V^T V as
 * produced by als_gramian.  A row with no stored entry gets X[u] = 0.  With
 * ALS_SOLVER_CG the rows of X in the range are also read (start vectors).  X must
 * have Y->rows rows, the same d and dtype as V, and must not overlap V.  All
 * arithmetic is fp32 (fp64 for the one shared d x d factorisation; products on the
 * bf16 matrix cores take fp32 operands as hi + lo bf16 parts, accurate to 2^-16, and
 * accumulate in fp32); the result is rounded once (to nearest even) to X's dtype.
 * With bf16 tables and d >= 32 the library's transformed copy of V (the table Z of
 * the k x k form) is kept in bf16 as well, one more rounding to the tables' own
 * element type (Section 4.4 keeps the tables in bf16 and the solve in fp32: the
 * solve stays fp32).  Rows outside the range are
 * left untouched.  Asynchronous on `stream`: nothing waits for the GPU and nothing
 * is copied back (the first call with a larger problem than any before grows the
 * workspace, which allocates).  A non-positive pivot sets a device flag reported as
 * ALS_ENOTSPD by the next als_loss/als_status_sync; an indptr that does not fit nnz
 * is reported there as ALS_EINVAL. */
als_status als_solve_rows(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                          const als_params *params, als_table *X, int64_t row_begin,
                          int64_t row_end, void *stream);

/* One epoch (Algorithm 1, one pass of the outer loop): G_H = H^T H; W <- rows of Y
 * solved against H; G_W = W^T W (from the new W); H <- rows of Yt solved against W.
 * Yt must be the transpose of Y in CSR form.  W and H are updated in place.
 * Once the workspace has reached its size (after the first call on a problem of this size) the call only
 * enqueues kernels - no allocation, no copy, no wait - and may be recorded into a HIP graph and replayed. */
als_status als_epoch(als_ctx *ctx, const als_csr *Y, const als_csr *Yt, als_table *W,
                     als_table *H, const als_params *params, void *stream);

/* The objective of Eq. 3,
 *     sum_{(u,i,y) in Y} (y - <w_u,h_i>)^2 + alpha * sum_u sum_i <w_u,h_i>^2
 *       + lambda * (||W||_F^2 + ||H||_F^2),
 * with the all-pairs term evaluated as <W^T W, H^T H>_F.  Writes one fp64 value
 * to host memory; synchronises `stream`. */
als_status als_loss(als_ctx *ctx, const als_csr *Y, const als_table *W, const als_table *H,
                    const als_params *params, double *loss_host, void *stream);

/* Exact top-k retrieval by inner product (the retrieval step of Section 4.6; with rows folded in by
 * als_solve_rows from part of their links it gives the Recall@K evaluation of Section 5):
 * for every row q of Q [nq x d] the k rows i of H [n x d] with the largest <Q[q], H[i]>, leaving out the
 * column ids stored in row q of `exclude` (nq rows, n columns; its values are not read; may be NULL).
 * ids: device int32 [nq*k], scores: device fp32 [nq*k], row q at offset q*k, best first, equal scores by
 * ascending id; where fewer than k rows are admissible the tail holds id -1 and score -inf.  Products and
 * sums are fp32 (bf16 tables are widened exactly).  1 <= k <= ALS_TOPK_MAX_K.  Asynchronous on `stream`. */
#define ALS_TOPK_MAX_K 64
als_status als_topk(als_ctx *ctx, const als_table *Q, const als_table *H, const als_csr *exclude, int32_t k,
                    int32_t *ids, float *scores, void *stream);

/* Synchronise `stream` and report (then clear) the device-side error flag. */
als_status als_status_sync(als_ctx *ctx, void *stream);

/* Opt-in validation pass over a CSR matrix (one pass over indptr and indices):
 * ALS_OK, or ALS_EINVAL if indptr is not monotone from 0 to nnz or a column id
 * is out of range.  Synchronises `stream`. */
als_status als_check_csr(als_ctx *ctx, const als_csr *Y, void *stream);

/* Diagnostics, not part of the method.  A plain device-to-device copy kernel of known size (`bytes`, a multiple of 16, both
 * pointers device and 16-byte aligned).  Hardware traffic counters (FETCH_SIZE, WRITE_SIZE) read for
 * this kernel give the scale factor applied to the counters of the other kernels. */
als_status als_copy_probe(als_ctx *ctx, const void *src, void *dst, int64_t bytes, void *stream);

/* Diagnostics, not part of the method.  GPU time in milliseconds (HIP events on the call's stream) of the
 * kernels launched by the most recent als_gramian / als_solve_rows / als_epoch / als_loss, per kernel:
 *   [0] Gramian (3 kernels)   [1] row classification (5 kernels)   [2] shared factorisation + Z = V L^-T
 *   [3] X = R L^-1   [4] primal fused row kernel   [5] long-row segment accumulation   [6] long-row reduce + solve
 *   [7] dual rows k <= 4   [8] dual rows 5 <= k <= 8   [9 + c] dual rows 16c < k <= 16(c+1), c = 0..7 (c = 0: 8 < k)
 * followed by the number of timed launches of each slot in [ALS_TIMING_SLOTS + slot].  Timing is recorded only
 * while enabled with als_set_timing(ctx, 1); reading waits for the recorded events. */
#define ALS_TIMING_SLOTS 17
als_status als_set_timing(als_ctx *ctx, int enabled);
als_status als_get_timing(als_ctx *ctx, double *ms_host /* [2 * ALS_TIMING_SLOTS] */);

const char *als_strerror(als_status status);
const char *als_last_error(const als_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* ALS_H */
