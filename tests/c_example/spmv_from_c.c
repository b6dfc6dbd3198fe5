/* Plain C user of the library: build a small CSR matrix (or read a Matrix Market file), let the
 * library pick a plan, run y = A*x on the GPU and check y against a loop written here.
 *
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude tests/c_example/spmv_from_c.c \
 *       -Lpaper_2212_10432_amd -lspmv_mi355 -L/opt/rocm/lib -lamdhip64 -lm -o spmv_from_c
 *   ./spmv_from_c [matrix.mtx]
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "spmv.h"

#define CHECK_HIP(call)                                                              \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));        \
            return 2;                                                                \
        }                                                                            \
    } while (0)
#define CHECK_SPMV(call)                                                             \
    do {                                                                             \
        spmv_status_t s_ = (call);                                                   \
        if (s_ != SPMV_OK) {                                                         \
            fprintf(stderr, "%s failed (%d): %s\n", #call, (int)s_, spmv_last_error()); \
            return 2;                                                                \
        }                                                                            \
    } while (0)

int main(int argc, char **argv) {
    int64_t nrows, ncols, nnz;
    int32_t *row_ptr, *col_idx;
    double *values;
    int from_file = argc > 1;
    if (from_file) {
        void *v = NULL;
        CHECK_SPMV(spmv_mm_read(argv[1], SPMV_F64, &nrows, &ncols, &nnz, &row_ptr, &col_idx, &v));
        values = (double *)v;
    } else { /* tridiagonal (2, -1) with a long first row */
        nrows = ncols = 5000;
        nnz = 3 * nrows - 2 + (ncols - 2);
        row_ptr = (int32_t *)malloc((size_t)(nrows + 1) * sizeof(int32_t));
        col_idx = (int32_t *)malloc((size_t)nnz * sizeof(int32_t));
        values = (double *)malloc((size_t)nnz * sizeof(double));
        int64_t k = 0;
        for (int64_t i = 0; i < nrows; ++i) {
            row_ptr[i] = (int32_t)k;
            if (i == 0) {
                for (int64_t j = 0; j < ncols; ++j) {
                    col_idx[k] = (int32_t)j;
                    values[k++] = j == 0 ? 2.0 : (j == 1 ? -1.0 : 0.5);
                }
                continue;
            }
            col_idx[k] = (int32_t)(i - 1), values[k++] = -1.0;
            col_idx[k] = (int32_t)i, values[k++] = 2.0;
            if (i + 1 < ncols) col_idx[k] = (int32_t)(i + 1), values[k++] = -1.0;
        }
        row_ptr[nrows] = (int32_t)k;
        nnz = k;
    }
    spmv_options_t opts = {0};
    opts.search_budget_ms = 500.0;
    spmv_plan_t *plan = NULL;
    CHECK_SPMV(spmv_plan_create(&plan, nrows, ncols, nnz, row_ptr, col_idx, values, SPMV_F64, &opts));
    size_t need = 0;
    CHECK_SPMV(spmv_plan_describe(plan, NULL, 0, &need));
    char *desc = (char *)malloc(need);
    CHECK_SPMV(spmv_plan_describe(plan, desc, need, NULL));
    printf("%.*s ...\n", 160, desc);

    double *x = (double *)malloc((size_t)ncols * sizeof(double));
    double *y = (double *)malloc((size_t)nrows * sizeof(double));
    for (int64_t j = 0; j < ncols; ++j) x[j] = 1.0 + (double)(j % 7) / 8.0;
    void *xd = NULL, *yd = NULL;
    CHECK_HIP(hipMalloc(&xd, (size_t)(ncols > 0 ? ncols : 1) * sizeof(double)));
    CHECK_HIP(hipMalloc(&yd, (size_t)(nrows > 0 ? nrows : 1) * sizeof(double)));
    CHECK_HIP(hipMemcpy(xd, x, (size_t)ncols * sizeof(double), hipMemcpyHostToDevice));
    CHECK_SPMV(spmv_run(plan, xd, yd, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(y, yd, (size_t)nrows * sizeof(double), hipMemcpyDeviceToHost));

    double worst = 0.0;
    for (int64_t i = 0; i < nrows; ++i) {
        double ref = 0.0, scale = 0.0;
        for (int64_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
            ref += values[k] * x[col_idx[k]];
            scale += fabs(values[k] * x[col_idx[k]]);
        }
        const double err = fabs(y[i] - ref) / (scale > 0 ? scale : 1.0);
        if (err > worst) worst = err;
    }
    printf("rows %lld, nnz %lld, worst |y - ref| / (|A||x|) = %.3g\n", (long long)nrows, (long long)nnz, worst);
    CHECK_SPMV(spmv_plan_destroy(plan));
    CHECK_HIP(hipFree(xd));
    CHECK_HIP(hipFree(yd));
    if (from_file) spmv_mm_free(row_ptr, col_idx, values);
    else free(row_ptr), free(col_idx), free(values);
    free(x), free(y), free(desc);
    return worst < 1e-12 ? 0 : 1;
}
