/*
 * Plain CSR sparse-dense products on the CPU -- the "classic sparse format"
 * computation the paper compares against (Section 2.2, text after Eq. (5):
 * nnz(A) scalar operations per column).  TEST / BASELINE INFRASTRUCTURE ONLY:
 * used by the tests and by the benchmark's CPU-baseline leg, never by the HIP
 * library, and it shares no code with it.
 *
 *   csr_spmm_f64      one thread, fp64 accumulation: Y[i,:] = sum_{j in a_i} X[j,:]
 *   csr_spmm_norm_f64 one thread, fp64: Y[i,:] = s_i * sum_{j in a_i v {i}} s_j X[j,:],
 *                     s = d^-1/2, d = row sums of A v I   (Eq. (1) text)
 *   csr_spmm_norm_omp_f32  all cores (OpenMP over rows), fp32 accumulation, inner
 *                     loop over k left to the compiler's vectoriser
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

void csr_spmm_f64(int64_t row_begin, int64_t row_end, const int64_t* rowptr, const int32_t* colidx,
                  const float* X, int64_t k, double* Y) {
    for (int64_t i = row_begin; i < row_end; ++i) {
        double* y = Y + (i - row_begin) * k;
        for (int64_t c = 0; c < k; ++c) y[c] = 0.0;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            const float* x = X + (int64_t)colidx[p] * k;
            for (int64_t c = 0; c < k; ++c) y[c] += (double)x[c];
        }
    }
}

void csr_spmm_norm_f64(int64_t row_begin, int64_t row_end, const int64_t* rowptr, const int32_t* colidx,
                       const int64_t* d, const float* X, int64_t k, double* Y) {
    for (int64_t i = row_begin; i < row_end; ++i) {
        double* y = Y + (i - row_begin) * k;
        int has_diag = 0;
        for (int64_t c = 0; c < k; ++c) y[c] = 0.0;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            const int64_t j = colidx[p];
            const double sj = 1.0 / sqrt((double)d[j]);
            const float* x = X + j * k;
            if (j == i) has_diag = 1;
            for (int64_t c = 0; c < k; ++c) y[c] += sj * (double)x[c];
        }
        const double si = 1.0 / sqrt((double)d[i]);
        if (!has_diag) {
            const float* x = X + i * k;
            for (int64_t c = 0; c < k; ++c) y[c] += si * (double)x[c];
        }
        for (int64_t c = 0; c < k; ++c) y[c] *= si;
    }
}

int csr_omp_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* s = d^-1/2 precomputed in fp32 by the caller; A v I taken with an explicit diagonal term */
void csr_spmm_norm_omp_f32(int64_t m, const int64_t* rowptr, const int32_t* colidx, const float* s,
                           const float* X, int64_t k, float* Y) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < m; ++i) {
        float* restrict y = Y + i * k;
        int has_diag = 0;
        for (int64_t c = 0; c < k; ++c) y[c] = 0.0f;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            const int64_t j = colidx[p];
            const float sj = s[j];
            const float* restrict x = X + j * k;
            if (j == i) has_diag = 1;
            for (int64_t c = 0; c < k; ++c) y[c] += sj * x[c];
        }
        if (!has_diag) {
            const float* restrict x = X + i * k;
            for (int64_t c = 0; c < k; ++c) y[c] += s[i] * x[c];
        }
        for (int64_t c = 0; c < k; ++c) y[c] *= s[i];
    }
}
