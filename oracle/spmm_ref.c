/*
 * CPU oracle for CSR sparse x dense multiplication.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  It is not part of the product: only the test-suite, the smoke
 * check and the "cpu_baseline" leg of the benchmark may build or call it, and
 * it shares no code (headers, helpers, constants) with the HIP sources.
 *
 * What it computes (paper Section 1, the problem statement Y = A X with A
 * sparse M x K, X dense K x N, Y dense M x N; N = 1 is SpMV):
 *
 *   Yref[i][n] = sum_{p = rowptr[i]}^{rowptr[i+1]-1} vals[p] * X[colidx[p]][n]
 *   Bnd [i][n] = sum_{p = rowptr[i]}^{rowptr[i+1]-1} |vals[p]| * |X[colidx[p]][n]|
 *
 * Inputs are fp32 (the paper's float2/float4 loads in Section 2.1.2 imply
 * single precision), every product and sum is taken in fp64 in increasing p,
 * and the result stays in fp64.  The paper's four kernels differ only in
 * schedule, never in the value computed, so the oracle is this definition
 * written out as three nested loops: rows, stored entries, dense columns.
 * X and Y are row-major with leading dimension N.  Column indices may appear
 * in any order inside a row; repeated (i,k) entries add.
 *
 * Bnd is the elementwise bound matrix |A| |X| that the acceptance test
 * |Y - Yref| <= tol * Bnd is written against.
 *
 * Rows are independent, so the optional OpenMP split over rows does not
 * change any result bit: each row is still summed by one thread in order.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Returns 0 on success, a positive code on a malformed matrix:
 *   1 = negative dimension, 2 = rowptr[0] != 0 or rowptr decreasing,
 *   3 = column index outside [0, K).
 * yref and bnd are M*N doubles each (bnd may be NULL to skip the bound).
 * nthreads <= 0 means "whatever OpenMP picks"; 1 forces the serial loop. */
int oracle_spmm_csr(int64_t M, int64_t K, int64_t N,
                    const int32_t *rowptr, const int32_t *colidx,
                    const float *vals, const float *X,
                    double *yref, double *bnd, int nthreads)
{
    if (M < 0 || K < 0 || N < 0)
        return 1;
    if (M == 0 || N == 0)
        return 0;
    if (rowptr[0] != 0)
        return 2;
    for (int64_t i = 0; i < M; ++i)
        if (rowptr[i + 1] < rowptr[i])
            return 2;
    for (int64_t p = 0; p < rowptr[M]; ++p)
        if (colidx[p] < 0 || colidx[p] >= K)
            return 3;

#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t i = 0; i < M; ++i) {
        double *yrow = yref + (size_t)i * (size_t)N;
        double *brow = bnd ? bnd + (size_t)i * (size_t)N : NULL;
        for (int64_t n = 0; n < N; ++n) {
            yrow[n] = 0.0;
            if (brow)
                brow[n] = 0.0;
        }
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            const double a = (double)vals[p];
            const float *xrow = X + (size_t)colidx[p] * (size_t)N;
            for (int64_t n = 0; n < N; ++n) {
                const double x = (double)xrow[n];
                yrow[n] += a * x;
                if (brow)
                    brow[n] += fabs(a) * fabs(x);
            }
        }
    }
    return 0;
}

/* Number of threads the parallel loop above will really use. */
int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
