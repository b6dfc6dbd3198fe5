/*
 * TEST ORACLE -- not part of the product.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may build or call this file.  It shares no code
 * with the GPU library.
 *
 * What it computes: sparse matrix-vector multiplication y = A*x (Section I of
 * the paper, first sentence: "SpMV, y=Ax") for A stored in CSR.  Every format
 * operator of the paper (Table II) is a re-layout of A or a re-association of
 * the per-row sums (Section IV-A), so the method's result has this plain
 * definition and the oracle is the definition written out:
 *
 *     y[i] = sum_{k = row_ptr[i]}^{row_ptr[i+1]-1} values[k] * x[col_idx[k]]
 *
 * with y[i] = +0 for an empty row; y is overwritten (alpha = 1, beta = 0).
 * The sum runs left to right in storage order.  Duplicate column indices in a
 * row simply add; columns need not be sorted.
 *
 * Variants:
 *   *_work : accumulate in the working precision (the literal definition)
 *   *_wide : accumulate in a wider type (long double for fp64 data, double for
 *            fp32 data -- an fp32*fp32 product is exact in double) and round
 *            once at the end; used as the centre of the tolerance test so the
 *            oracle's own rounding on 100,000-entry rows does not use up the
 *            1e-12 / 1e-5 budget
 *   abs_*  : (|A| |x|)_i in the wide type -- the scale of the tolerance
 *
 * `threads` > 1 distributes whole rows over OpenMP threads (each row is still
 * summed sequentially by one thread); it changes no result.
 *
 * Build:  gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC csr_spmv_ref.c -o liboracle.so
 */
#include <stdint.h>
#include <math.h>

#define ROW_LOOP(ACC_T, OUT_T, EXPR)                                            \
    _Pragma("omp parallel for schedule(static) num_threads(threads)")          \
    for (int64_t i = 0; i < nrows; ++i) {                                       \
        ACC_T acc = 0;                                                          \
        for (int64_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) acc += EXPR;      \
        y[i] = (OUT_T)acc;                                                      \
    }

void csr_spmv_f64_work(int64_t nrows, const int32_t *row_ptr, const int32_t *col_idx,
                       const double *values, const double *x, double *y, int threads) {
    if (threads < 1) threads = 1;
    ROW_LOOP(double, double, values[k] * x[col_idx[k]])
}

void csr_spmv_f32_work(int64_t nrows, const int32_t *row_ptr, const int32_t *col_idx,
                       const float *values, const float *x, float *y, int threads) {
    if (threads < 1) threads = 1;
    ROW_LOOP(float, float, values[k] * x[col_idx[k]])
}

void csr_spmv_f64_wide(int64_t nrows, const int32_t *row_ptr, const int32_t *col_idx,
                       const double *values, const double *x, double *y, int threads) {
    if (threads < 1) threads = 1;
    ROW_LOOP(long double, double, (long double)values[k] * (long double)x[col_idx[k]])
}

/* fp32 data, double accumulation, double output (not rounded back to fp32) */
void csr_spmv_f32_wide(int64_t nrows, const int32_t *row_ptr, const int32_t *col_idx,
                       const float *values, const float *x, double *y, int threads) {
    if (threads < 1) threads = 1;
    ROW_LOOP(double, double, (double)values[k] * (double)x[col_idx[k]])
}

void csr_abs_f64(int64_t nrows, const int32_t *row_ptr, const int32_t *col_idx,
                 const double *values, const double *x, double *y, int threads) {
    if (threads < 1) threads = 1;
    ROW_LOOP(long double, double, fabsl((long double)values[k]) * fabsl((long double)x[col_idx[k]]))
}

void csr_abs_f32(int64_t nrows, const int32_t *row_ptr, const int32_t *col_idx,
                 const float *values, const float *x, double *y, int threads) {
    if (threads < 1) threads = 1;
    ROW_LOOP(double, double, fabs((double)values[k]) * fabs((double)x[col_idx[k]]))
}
