/*
 * CPU oracle for the implicit-ALS half-epoch (TEST INFRASTRUCTURE, not product code).
 *
 * A plain, slow, fp64 implementation of what the GPU library computes, written
 * straight from the paper's problem statement: the objective (Section 3, Eq. 3),
 * the closed-form row update (Eq. 4) and the loop structure of Algorithm 1.
 * It shares no code with the HIP path and is only ever called from tests, the
 * smoke check and the benchmark's CPU-baseline leg.
 *
 * Conventions: tables are row-major fp64 [rows x d] (the caller widens fp32 or
 * bf16 storage exactly); the sparse matrix is CSR with int64 indptr, int32
 * column ids and optional fp32 labels (NULL means y = 1 for every stored
 * entry).  Parallelism: OpenMP over rows only; no blocking, no reordering.
 *
 * Pins (tests/test_oracle_pins.py): brute-force least squares, zero gradient
 * with the literal all-pairs sum, monotone objective, closed forms (empty row,
 * single entry via Sherman-Morrison, d = 1, identity table, alpha = 0 ridge),
 * structural invariants, trace-form loss vs literal double sum.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ENOTSPD 5
#define ORACLE_ENOMEM 6

/* Round an fp64 value to the storage precision of a table entry.
 * storage: 0 = keep fp64, 1 = fp32 (round to nearest even, as the C cast does),
 *          2 = bfloat16 (round to nearest even on the fp32 bit pattern).
 * Section 4.4: the solution is cast back to the table's precision on store. */
static double round_storage(double x, int storage) {
    if (storage == 0) return x;
    float f = (float)x;
    if (storage == 1) return (double)f;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) != 0x7f800000u) {          /* finite */
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
    }
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

void oracle_round_storage(double *x, int64_t count, int storage) {
    for (int64_t i = 0; i < count; ++i) x[i] = round_storage(x[i], storage);
}

/* G = V^T V  (Algorithm 1, line 2; Section 3 after Eq. 4). */
int oracle_gramian(const double *V, int64_t n, int d, double *G) {
    for (int a = 0; a < d * d; ++a) G[a] = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        const double *v = V + j * d;
        for (int a = 0; a < d; ++a)
            for (int b = 0; b < d; ++b) G[a * d + b] += v[a] * v[b];
    }
    return ORACLE_OK;
}

/* In-place Cholesky A = L L^T on the lower triangle, then solve A x = b.
 * Returns nonzero if a pivot is not positive. */
static int chol_solve(double *A, double *b, int d) {
    for (int k = 0; k < d; ++k) {
        double s = A[k * d + k];
        for (int p = 0; p < k; ++p) s -= A[k * d + p] * A[k * d + p];
        if (!(s > 0.0)) return ORACLE_ENOTSPD;
        double lkk = sqrt(s);
        A[k * d + k] = lkk;
        for (int i = k + 1; i < d; ++i) {
            double t = A[i * d + k];
            for (int p = 0; p < k; ++p) t -= A[i * d + p] * A[k * d + p];
            A[i * d + k] = t / lkk;
        }
    }
    for (int i = 0; i < d; ++i) {                     /* L z = b */
        double t = b[i];
        for (int p = 0; p < i; ++p) t -= A[i * d + p] * b[p];
        b[i] = t / A[i * d + i];
    }
    for (int i = d - 1; i >= 0; --i) {                /* L^T x = z */
        double t = b[i];
        for (int p = i + 1; p < d; ++p) t -= A[p * d + i] * b[p];
        b[i] = t / A[i * d + i];
    }
    return ORACLE_OK;
}

/* The row update of Eq. 4 / Algorithm 1 lines 3-10 for a list of rows.
 *   A = alpha*G + lambda*I ; b = 0
 *   for every stored (u, i, y):  b += y * V[i] ;  A += V[i] (x) V[i]
 *   X[u] = A^{-1} b, rounded once to the storage precision.
 * row_ids == NULL means rows 0..nrows-1.  X is [nrows x d], row r of X holds
 * the solution for row_ids[r]. */
int oracle_solve_rows(const int64_t *indptr, const int32_t *indices, const float *values,
                      const double *V, int d, const double *G, double alpha, double lambda,
                      const int64_t *row_ids, int64_t nrows, int storage, double *X) {
    int status = ORACLE_OK;
#pragma omp parallel
    {
        double *A = (double *)malloc(sizeof(double) * (size_t)d * d);
        double *b = (double *)malloc(sizeof(double) * (size_t)d);
        if (!A || !b) {
#pragma omp critical
            status = ORACLE_ENOMEM;
        } else {
#pragma omp for schedule(dynamic, 64)
            for (int64_t r = 0; r < nrows; ++r) {
                int64_t u = row_ids ? row_ids[r] : r;
                for (int a = 0; a < d; ++a) {
                    b[a] = 0.0;
                    for (int c = 0; c < d; ++c) A[a * d + c] = alpha * G[a * d + c] + (a == c ? lambda : 0.0);
                }
                for (int64_t p = indptr[u]; p < indptr[u + 1]; ++p) {
                    const double *h = V + (int64_t)indices[p] * d;
                    double y = values ? (double)values[p] : 1.0;
                    for (int a = 0; a < d; ++a) {
                        b[a] += y * h[a];
                        for (int c = 0; c < d; ++c) A[a * d + c] += h[a] * h[c];
                    }
                }
                int rc = chol_solve(A, b, d);
                if (rc != ORACLE_OK) {
#pragma omp critical
                    status = rc;
                }
                for (int a = 0; a < d; ++a) X[r * d + a] = round_storage(b[a], storage);
            }
        }
        free(A);
        free(b);
    }
    return status;
}

/* One half-epoch: Gramian of the fixed side, then every row of Y solved. */
int oracle_half_epoch(const int64_t *indptr, const int32_t *indices, const float *values,
                      int64_t m, int64_t n, const double *V, int d, double alpha, double lambda,
                      int storage, double *X) {
    double *G = (double *)malloc(sizeof(double) * (size_t)d * d);
    if (!G) return ORACLE_ENOMEM;
    oracle_gramian(V, n, d, G);
    int rc = oracle_solve_rows(indptr, indices, values, V, d, G, alpha, lambda, NULL, m, storage, X);
    free(G);
    return rc;
}

/* One epoch (Algorithm 1, one pass of the outer loop): solve W against H over Y,
 * then H against the NEW W over Y^T.  W [m x d] and H [n x d] are updated in place. */
int oracle_epoch(const int64_t *indptr, const int32_t *indices, const float *values,
                 const int64_t *t_indptr, const int32_t *t_indices, const float *t_values,
                 int64_t m, int64_t n, int d, double alpha, double lambda, int storage,
                 double *W, double *H) {
    int rc = oracle_half_epoch(indptr, indices, values, m, n, H, d, alpha, lambda, storage, W);
    if (rc != ORACLE_OK) return rc;
    return oracle_half_epoch(t_indptr, t_indices, t_values, n, m, W, d, alpha, lambda, storage, H);
}

/* Observed part of Eq. 3: sum over stored entries of (y - <w_u, h_i>)^2. */
double oracle_loss_observed(const int64_t *indptr, const int32_t *indices, const float *values,
                            int64_t m, const double *W, const double *H, int d) {
    double total = 0.0;
#pragma omp parallel for reduction(+ : total) schedule(dynamic, 256)
    for (int64_t u = 0; u < m; ++u) {
        for (int64_t p = indptr[u]; p < indptr[u + 1]; ++p) {
            const double *h = H + (int64_t)indices[p] * d;
            double dot = 0.0;
            for (int a = 0; a < d; ++a) dot += W[u * d + a] * h[a];
            double y = values ? (double)values[p] : 1.0;
            total += (y - dot) * (y - dot);
        }
    }
    return total;
}

/* Eq. 3 with the all-pairs term evaluated through the Gramians:
 *   sum_u sum_i <w_u,h_i>^2 = sum_{a,b} (W^T W)_{ab} (H^T H)_{ab}. */
double oracle_loss(const int64_t *indptr, const int32_t *indices, const float *values,
                   int64_t m, int64_t n, const double *W, const double *H, int d,
                   double alpha, double lambda) {
    double *GW = (double *)malloc(sizeof(double) * (size_t)d * d);
    double *GH = (double *)malloc(sizeof(double) * (size_t)d * d);
    if (!GW || !GH) { free(GW); free(GH); return NAN; }
    oracle_gramian(W, m, d, GW);
    oracle_gramian(H, n, d, GH);
    double pairs = 0.0, norms = 0.0;
    for (int a = 0; a < d * d; ++a) pairs += GW[a] * GH[a];
    for (int a = 0; a < d; ++a) norms += GW[a * d + a] + GH[a * d + a];
    free(GW);
    free(GH);
    return oracle_loss_observed(indptr, indices, values, m, W, H, d) + alpha * pairs + lambda * norms;
}

/* Eq. 3 exactly as printed: the all-pairs term as a double sum over every (u, i).
 * O(m n d): tiny inputs only. */
double oracle_loss_literal(const int64_t *indptr, const int32_t *indices, const float *values,
                           int64_t m, int64_t n, const double *W, const double *H, int d,
                           double alpha, double lambda) {
    double pairs = 0.0, norms = 0.0;
    for (int64_t u = 0; u < m; ++u)
        for (int64_t i = 0; i < n; ++i) {
            double dot = 0.0;
            for (int a = 0; a < d; ++a) dot += W[u * d + a] * H[i * d + a];
            pairs += dot * dot;
        }
    for (int64_t u = 0; u < m * d; ++u) norms += W[u] * W[u];
    for (int64_t i = 0; i < n * d; ++i) norms += H[i] * H[i];
    return oracle_loss_observed(indptr, indices, values, m, W, H, d) + alpha * pairs + lambda * norms;
}

int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
