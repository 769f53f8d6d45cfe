/*
 * CPU oracle for CSR SpMV  y = A x.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product library may call, link or include this file.
 *
 * Every load-balancing schedule of the case study (Table II: thread-, wavefront-,
 * block-mapped, work-oriented/merge-path) computes the same inner-product SpMV
 * (Sec. IV), so the oracle is that definition written out: for each row i,
 *
 *     y_ref[i] = sum_{k = row_ptr[i]}^{row_ptr[i+1]-1} values[k] * x[col_idx[k]]
 *     bound[i] = sum_{k}                               |values[k]| * |x[col_idx[k]]|
 *
 * accumulated left to right in fp64.  (fp32 inputs; every product of two fp32
 * numbers is exact in fp64.)  bound[] is what the fp32 tolerance
 * |y - y_ref| <= 1e-5 * bound is measured against.
 *
 * Plain C, one thread, no blocking, no vectorisation hints.
 */
#include <math.h>
#include <stdint.h>

void oracle_spmv_f64(int64_t rows, const int32_t *row_ptr, const int32_t *col_idx,
                     const float *values, const float *x, double *y_ref, double *bound)
{
    for (int64_t i = 0; i < rows; ++i) {
        double s = 0.0, b = 0.0;
        for (int64_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
            double p = (double)values[k] * (double)x[col_idx[k]];
            s += p;
            b += fabs(p);
        }
        y_ref[i] = s;
        if (bound) bound[i] = b;
    }
}

/* Same loop without the bound, the form that is timed as the CPU baseline. */
void oracle_spmv_f64_nobound(int64_t rows, const int32_t *row_ptr, const int32_t *col_idx,
                             const float *values, const float *x, double *y_ref)
{
    for (int64_t i = 0; i < rows; ++i) {
        double s = 0.0;
        for (int64_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k)
            s += (double)values[k] * (double)x[col_idx[k]];
        y_ref[i] = s;
    }
}
