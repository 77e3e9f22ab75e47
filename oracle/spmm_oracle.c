/*
 * CPU oracle for C = A * B  (TEST INFRASTRUCTURE, not part of the product path).
 *
 * Definition followed: the paper's problem statement in Section 2 ("Background"),
 * A (n x n, sparse, CSR) times B (n x dim, dense) = C (n x dim), together with the
 * inner loop of Algorithm 1: every stored nonzero (i, j, a_ij) contributes
 * a_ij * B[j][k] to C[i][k].  PCSR, vector size, balancing and coarsening only
 * change how the work is laid out, never the result, so the oracle works straight
 * from the input CSR arrays and knows nothing about PCSR.
 *
 * Arithmetic: each fp32 operand is widened to fp64, the product and the running sum
 * are fp64, nonzeros of a row are taken in stored order.  Alongside C the oracle
 * returns bound[i][k] = sum_j |a_ij * B[j][k]|, the scale of the admissible error
 * |C_gpu - C_ref| <= 1e-5 * bound + 1e-6.
 *
 * Rows are independent, so an OpenMP parallel-for over rows changes no arithmetic.
 * Only tests/, the smoke check and the bench's cpu_baseline leg may call this.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* One output row: C_row[k] and bound_row[k] for k in [0, K). */
static void oracle_row(const int32_t *rowptr, const int32_t *colidx, const float *vals,
                       const float *B, int64_t K, int64_t i, double *C_row, double *bound_row)
{
    for (int64_t k = 0; k < K; ++k) {
        C_row[k] = 0.0;
        if (bound_row) bound_row[k] = 0.0;
    }
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
        const double a = (double)vals[p];
        const float *b_row = B + (int64_t)colidx[p] * K;
        for (int64_t k = 0; k < K; ++k) {
            const double term = a * (double)b_row[k];
            C_row[k] += term;
            if (bound_row) bound_row[k] += fabs(term);
        }
    }
}

/* Full product.  C and bound are n_rows x K row-major fp64; bound may be NULL. */
int oracle_spmm_csr(int64_t n_rows, const int32_t *rowptr, const int32_t *colidx,
                    const float *vals, const float *B, int64_t K, double *C, double *bound,
                    int32_t n_threads)
{
    if (n_rows < 0 || K < 0 || !rowptr || !C) return -1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_rows; ++i)
        oracle_row(rowptr, colidx, vals, B, K, i, C + i * K, bound ? bound + i * K : NULL);
    return 0;
}

/* Selected rows only: output row r holds C[rows[r]][:] (n_sel x K). */
int oracle_spmm_csr_rows(const int32_t *rowptr, const int32_t *colidx, const float *vals,
                         const float *B, int64_t K, const int64_t *rows, int64_t n_sel,
                         double *C, double *bound, int32_t n_threads)
{
    if (n_sel < 0 || K < 0 || !rowptr || !rows || !C) return -1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t r = 0; r < n_sel; ++r)
        oracle_row(rowptr, colidx, vals, B, K, rows[r], C + r * K, bound ? bound + r * K : NULL);
    return 0;
}

/* Number of threads a parallel region would use (reported beside timings). */
int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
