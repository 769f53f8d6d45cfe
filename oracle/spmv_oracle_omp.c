/*
 * The CPU oracle's row loop for y = A x (Sec. IV: every schedule computes the same
 * inner-product SpMV) with the rows shared out among all host threads.  TEST
 * INFRASTRUCTURE ONLY, and only a timed baseline: the value checked against is always the
 * single-thread loop of spmv_oracle.c, which this one must equal bit for bit (each row is
 * still summed left to right in fp64 by one thread).  Nothing in the product library may
 * call, link or include this file.
 */
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_spmv_f64_all_cores(int64_t rows, const int32_t *row_ptr, const int32_t *col_idx,
                              const float *values, const float *x, double *y_ref)
{
    int threads = 1;
#pragma omp parallel
    {
#pragma omp single
        {
#ifdef _OPENMP
            threads = omp_get_num_threads();
#endif
        }
#pragma omp for schedule(static)
        for (int64_t i = 0; i < rows; ++i) {
            double s = 0.0;
            for (int64_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k)
                s += (double)values[k] * (double)x[col_idx[k]];
            y_ref[i] = s;
        }
    }
    return threads;
}
