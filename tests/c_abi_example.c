/*
 * A C caller of libdgsp: no C++, no Python, only the C-ABI of include/dgsp.h
 * and the HIP runtime for device memory.  Builds a small banded matrix on the
 * host, multiplies it by a dense matrix on the GPU with each of the four
 * kernels and with the adaptive call, and compares with a plain host loop.
 * Exit code 0 = every result within 1e-5 * (|A| |X|) of the host loop.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../include/dgsp.h"

#define CHECK_HIP(call)                                                            \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) {                                                    \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));      \
            return 2;                                                              \
        }                                                                          \
    } while (0)

int main(void) {
    const int64_t M = 3000, K = 3000, N = 4;
    /* row i holds columns i-2..i+2 (inside the matrix) except that every 7th row is empty */
    int32_t *rowptr = (int32_t *)malloc((size_t)(M + 1) * sizeof(int32_t));
    int32_t *colidx = (int32_t *)malloc((size_t)M * 5 * sizeof(int32_t));
    float *vals = (float *)malloc((size_t)M * 5 * sizeof(float));
    float *X = (float *)malloc((size_t)(K * N) * sizeof(float));
    double *ref = (double *)calloc((size_t)(M * N), sizeof(double));
    double *bnd = (double *)calloc((size_t)(M * N), sizeof(double));
    float *Y = (float *)malloc((size_t)(M * N) * sizeof(float));
    if (!rowptr || !colidx || !vals || !X || !ref || !bnd || !Y) return 2;
    int64_t nnz = 0;
    rowptr[0] = 0;
    for (int64_t i = 0; i < M; ++i) {
        if (i % 7 != 3) {
            for (int64_t c = i - 2; c <= i + 2; ++c) {
                if (c < 0 || c >= K) continue;
                colidx[nnz] = (int32_t)c;
                vals[nnz] = (float)(((i * 31 + c * 17) % 23) - 11) / 8.0f;
                ++nnz;
            }
        }
        rowptr[i + 1] = (int32_t)nnz;
    }
    for (int64_t k = 0; k < K * N; ++k) X[k] = (float)((k * 37) % 19 - 9) / 4.0f;
    for (int64_t i = 0; i < M; ++i)
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p)
            for (int64_t n = 0; n < N; ++n) {
                const double t = (double)vals[p] * (double)X[(int64_t)colidx[p] * N + n];
                ref[i * N + n] += t;
                bnd[i * N + n] += fabs(t);
            }

    dgsp_features_t feat;
    if (dgsp_features_from_csr_host(M, K, rowptr, colidx, &feat) != DGSP_OK) return 3;
    printf("features: nnz %lld avg_row %.3f cv_row %.3f max_row %lld -> rules pick %s for N = %lld\n",
           (long long)feat.nnz, feat.avg_row, feat.cv_row, (long long)feat.max_row,
           dgsp_algo_name(dgsp_select_algo(&feat, N)), (long long)N);

    int32_t *d_rowptr, *d_colidx;
    float *d_vals, *d_X, *d_Y;
    CHECK_HIP(hipMalloc((void **)&d_rowptr, (size_t)(M + 1) * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void **)&d_colidx, (size_t)nnz * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void **)&d_vals, (size_t)nnz * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&d_X, (size_t)(K * N) * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&d_Y, (size_t)(M * N) * sizeof(float)));
    CHECK_HIP(hipMemcpy(d_rowptr, rowptr, (size_t)(M + 1) * sizeof(int32_t), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_colidx, colidx, (size_t)nnz * sizeof(int32_t), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_vals, vals, (size_t)nnz * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_X, X, (size_t)(K * N) * sizeof(float), hipMemcpyHostToDevice));

    int failures = 0;
    for (int algo = DGSP_AUTO; algo <= DGSP_NB_PR; ++algo) {
        CHECK_HIP(hipMemset(d_Y, 0xff, (size_t)(M * N) * sizeof(float)));      /* NaN bit patterns */
        int chosen = algo;
        const int rc = algo == DGSP_AUTO
            ? dgsp_spmm_csr_auto(M, K, N, &feat, d_rowptr, d_colidx, d_vals, d_X, d_Y, &chosen, NULL)
            : dgsp_spmm_csr(M, K, N, d_rowptr, d_colidx, d_vals, d_X, d_Y, algo, NULL);
        if (rc != DGSP_OK) {
            fprintf(stderr, "%s: %s\n", dgsp_algo_name(algo), dgsp_status_string(rc));
            return 4;
        }
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(Y, d_Y, (size_t)(M * N) * sizeof(float), hipMemcpyDeviceToHost));
        double worst = 0.0;
        int bad = 0;
        for (int64_t e = 0; e < M * N; ++e) {
            const double err = fabs((double)Y[e] - ref[e]);
            if (!(err <= 1e-5 * bnd[e])) ++bad;                 /* also catches NaN; bnd == 0 demands exact 0 */
            if (bnd[e] > 0 && err / bnd[e] > worst) worst = err / bnd[e];
        }
        printf("%-6s%s worst |err|/(|A||X|) = %.2e  %s\n", algo == DGSP_AUTO ? "auto" : dgsp_algo_name(algo),
               algo == DGSP_AUTO ? (chosen == DGSP_RS_SR ? " (rs_sr)" : chosen == DGSP_RS_PR ? " (rs_pr)"
                                    : chosen == DGSP_NB_SR ? " (nb_sr)" : " (nb_pr)") : "        ",
               worst, bad ? "FAIL" : "ok");
        failures += bad != 0;
    }
    (void)hipFree(d_rowptr); (void)hipFree(d_colidx); (void)hipFree(d_vals); (void)hipFree(d_X); (void)hipFree(d_Y);
    free(rowptr); free(colidx); free(vals); free(X); free(ref); free(bnd); free(Y);
    return failures ? 1 : 0;
}
