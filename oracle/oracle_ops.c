/*
 * oracle_ops.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain, slow CPU operators that the unfused ("Base") plans of the paper's
 * four fusion examples (Fig. 1a-1d; Sec. 5.2 "Operations Performance") are
 * built from.  Every routine is ONE basic operator: it makes one pass over its
 * inputs and writes a freshly materialised output, exactly what fusion removes
 * (Sec. 1, "Fusion Opportunities").  Nothing here is blocked, fused or
 * reordered beyond what the operator's definition states.
 *
 * Precision: the paper computes in FP64 (Sec. 5.1, "Baselines").  Inputs and
 * outputs are doubles.  Every *accumulation* is carried in x87 extended
 * precision (64-bit significand) so that this side of a comparison is the more
 * accurate one: the paper fixes no summation order, so any order is a correct
 * result and the checker should not add rounding noise of its own.
 *
 * Parallelism: optional OpenMP over fixed-size chunks; chunk boundaries and
 * the order in which chunk partials are combined never depend on the number
 * of threads, so results are identical at any thread count.
 *
 * Nothing in this file is shared with, included by, or derived from the GPU
 * library; only tests, the smoke check and the benchmark's cpu_baseline leg
 * may load it.
 */
#include <float.h>
#include <stdint.h>
#include <stddef.h>

#if LDBL_MANT_DIG < 64
#error "oracle_ops.c expects long double with a >= 64-bit significand (x86-64)"
#endif

#ifdef _OPENMP
#include <omp.h>
#endif

typedef long double acc_t;

#define CHUNK ((int64_t)1 << 16)

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- sums --- */

/* sum(A): full aggregate of a contiguous array of n doubles (Fig. 1a, 1c). */
double oracle_sum(const double *a, int64_t n)
{
    int64_t nchunks = (n + CHUNK - 1) / CHUNK;
    acc_t total = 0.0L;
    /* chunk partials are combined strictly in chunk order */
#pragma omp parallel for ordered schedule(static, 1)
    for (int64_t c = 0; c < nchunks; ++c) {
        int64_t lo = c * CHUNK, hi = lo + CHUNK < n ? lo + CHUNK : n;
        acc_t s = 0.0L;
        for (int64_t i = lo; i < hi; ++i)
            s += (acc_t)a[i];
#pragma omp ordered
        total += s;
    }
    return (double)total;
}

/* rowSums(A): out[i] = sum_j A[i, j]; A is m x n row-major with leading dimension ld. */
void oracle_row_sums(const double *a, int64_t m, int64_t n, int64_t ld, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        acc_t s = 0.0L;
        for (int64_t j = 0; j < n; ++j)
            s += (acc_t)a[i * ld + j];
        out[i] = (double)s;
    }
}

/* colSums(A): out[j] = sum_i A[i, j]. */
void oracle_col_sums(const double *a, int64_t m, int64_t n, int64_t ld, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        acc_t s = 0.0L;
        for (int64_t i = 0; i < m; ++i)
            s += (acc_t)a[i * ld + j];
        out[j] = (double)s;
    }
}

/* ------------------------------------------------- dense matrix-vector --- */

/* q = X %*% v  (first product of Fig. 1b): q[i] = sum_j X[i,j] v[j]. */
void oracle_matvec(const double *x, int64_t m, int64_t n, int64_t ld,
                   const double *v, double *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        acc_t s = 0.0L;
        for (int64_t j = 0; j < n; ++j)
            s += (acc_t)x[i * ld + j] * (acc_t)v[j];
        q[i] = (double)s;
    }
}

/* out = t(X) %*% q  (second product of Fig. 1b, a second scan of X):
 * out[j] = sum_i X[i,j] q[i]. */
void oracle_t_matvec(const double *x, int64_t m, int64_t n, int64_t ld,
                     const double *q, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        acc_t s = 0.0L;
        for (int64_t i = 0; i < m; ++i)
            s += (acc_t)x[i * ld + j] * (acc_t)q[i];
        out[j] = (double)s;
    }
}

/* ------------------------------------------------------------ CSR ops ---- */
/* CSR: rowptr has m+1 int64 entries, colidx int32, vals double; every STORED
 * entry is processed (the Outer/sparse-Row binding is to the stored cells). */

/* q = X %*% v for CSR X. */
void oracle_csr_matvec(const int64_t *rowptr, const int32_t *colidx, const double *vals,
                       int64_t m, const double *v, double *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        acc_t s = 0.0L;
        for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
            s += (acc_t)vals[k] * (acc_t)v[colidx[k]];
        q[i] = (double)s;
    }
}

/* out = t(X) %*% q for CSR X: out[j] = sum over stored (i,j) of X[i,j] q[i].
 * Sequential over rows so that the accumulation order is the row order. */
void oracle_csr_t_matvec(const int64_t *rowptr, const int32_t *colidx, const double *vals,
                         int64_t m, int64_t n, const double *q, double *out, acc_t *work)
{
    for (int64_t j = 0; j < n; ++j)
        work[j] = 0.0L;
    for (int64_t i = 0; i < m; ++i) {
        acc_t qi = (acc_t)q[i];
        for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
            work[colidx[k]] += (acc_t)vals[k] * qi;
    }
    for (int64_t j = 0; j < n; ++j)
        out[j] = (double)work[j];
}

size_t oracle_acc_size(void) { return sizeof(acc_t); }

/* P_k = U[i_k,:] . V[j_k,:] for every stored cell k = (i_k, j_k) of CSR X
 * (the per-non-zero inner product w_ij of Sec. 2.2, "Code Generation").
 * U is m x r (ld ldu), V is n x r (ld ldv); p has nnz entries. */
void oracle_csr_uv_dot(const int64_t *rowptr, const int32_t *colidx, int64_t m,
                       const double *u, int64_t ldu, const double *v, int64_t ldv,
                       int64_t r, double *p)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < m; ++i) {
        for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
            const double *ui = u + i * ldu;
            const double *vj = v + (int64_t)colidx[k] * ldv;
            acc_t s = 0.0L;
            for (int64_t t = 0; t < r; ++t)
                s += (acc_t)ui[t] * (acc_t)vj[t];
            p[k] = (double)s;
        }
    }
}

/* D = U %*% t(V), dense m x n (what the Base plan of Fig. 1d materialises). */
void oracle_matmul_nt(const double *u, int64_t m, int64_t ldu, const double *v, int64_t n,
                      int64_t ldv, int64_t r, double *d)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            acc_t s = 0.0L;
            for (int64_t t = 0; t < r; ++t)
                s += (acc_t)u[i * ldu + t] * (acc_t)v[j * ldv + t];
            d[i * n + j] = (double)s;
        }
}

/* Row-segment sums over the stored cells of a CSR pattern:
 * out[i] = sum_{k in row i} a[k].  (rowSums of a matrix that has X's pattern.) */
void oracle_csr_row_sums(const int64_t *rowptr, int64_t m, const double *a, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        acc_t s = 0.0L;
        for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
            s += (acc_t)a[k];
        out[i] = (double)s;
    }
}

/* Column sums over the stored cells of a CSR pattern: out[j] = sum_{k: col k = j} a[k]. */
void oracle_csr_col_sums(const int64_t *rowptr, const int32_t *colidx, int64_t m, int64_t n,
                         const double *a, double *out, acc_t *work)
{
    for (int64_t j = 0; j < n; ++j)
        work[j] = 0.0L;
    for (int64_t k = 0; k < rowptr[m]; ++k)
        work[colidx[k]] += (acc_t)a[k];
    for (int64_t j = 0; j < n; ++j)
        out[j] = (double)work[j];
}

/* O = W %*% B for a matrix W stored on a CSR pattern (w = its nnz values) and
 * dense B (n x r, ld ldb): O[i,:] = sum over stored (i,j) of w_ij * B[j,:].
 * With B = V this is the right-hand Outer product of Sec. 2.2 ("scale V_j by
 * w_ij and add it to the output row I_i").  O is m x r, contiguous. */
void oracle_csr_matmul_dense(const int64_t *rowptr, const int32_t *colidx, const double *w,
                             int64_t m, const double *b, int64_t ldb, int64_t r, double *o)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t t = 0; t < r; ++t) {
            acc_t s = 0.0L;
            for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
                s += (acc_t)w[k] * (acc_t)b[(int64_t)colidx[k] * ldb + t];
            o[i * r + t] = (double)s;
        }
}

/* O = t(W) %*% B for W on a CSR pattern (m rows, n columns) and dense B (m x r):
 * O[j,:] = sum over stored (i,j) of w_ij * B[i,:]  (the left-hand Outer product).
 * O is n x r, contiguous; work holds n*r extended-precision accumulators. */
void oracle_csr_t_matmul_dense(const int64_t *rowptr, const int32_t *colidx, const double *w,
                               int64_t m, int64_t n, const double *b, int64_t ldb, int64_t r,
                               double *o, acc_t *work)
{
    for (int64_t x = 0; x < n * r; ++x)
        work[x] = 0.0L;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
            acc_t wk = (acc_t)w[k];
            acc_t *dst = work + (int64_t)colidx[k] * r;
            for (int64_t t = 0; t < r; ++t)
                dst[t] += wk * (acc_t)b[i * ldb + t];
        }
    for (int64_t x = 0; x < n * r; ++x)
        o[x] = (double)work[x];
}

/* C = A %*% B for dense A (m x n, ld lda) and B (n x k, ld ldb); C is m x k, contiguous.
 * (X %*% V of the matrix-matrix chain of Fig. 8g; vectMatMult per row.) */
void oracle_matmul(const double *a, int64_t m, int64_t n, int64_t lda, const double *b, int64_t k,
                   int64_t ldb, double *c)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < k; ++j) {
            acc_t s = 0.0L;
            for (int64_t t = 0; t < n; ++t)
                s += (acc_t)a[i * lda + t] * (acc_t)b[t * ldb + j];
            c[i * k + j] = (double)s;
        }
}

/* C = t(A) %*% Q for dense A (m x n, ld lda) and Q (m x k, ld ldq); C is n x k, contiguous.
 * (t(X) %*% (...) of Fig. 8g and of the multinomial-logistic-regression core, Sec. 2.2, second
 * example expression; vectOuterMultAdd per row.) */
void oracle_t_matmul(const double *a, int64_t m, int64_t n, int64_t lda, const double *q, int64_t k,
                     int64_t ldq, double *c)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t)
        for (int64_t j = 0; j < k; ++j) {
            acc_t s = 0.0L;
            for (int64_t i = 0; i < m; ++i)
                s += (acc_t)a[i * lda + t] * (acc_t)q[i * ldq + j];
            c[t * k + j] = (double)s;
        }
}
