/*
 * CPU oracle for batch-1 SpMV  y = W x  -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may call this.  It shares
 * no code with the EC-CSR encoder or the HIP kernels.
 *
 * What it computes (paper, Section 1: the kernel in question is the product of the sparse
 * weight matrix W with the input vector; Section 2.1: W has shape (M, K); Section 2.2: the
 * batch size is 1, so the input is a vector):
 *
 *     y[i] = sum_{j=0}^{n-1} W[i,j] * x[j]        S[i] = sum_j |W[i,j] * x[j]|
 *
 * taken directly from the DENSE masked FP16 matrix: every FP16 input is converted
 * exactly to FP64, products and sums are FP64, columns are visited in natural order
 * j = 0, 1, ..., n-1.  No sparse format, no blocking, no reordering.  S is the magnitude
 * the acceptance band  |y - y_ref| <= 2e-3 * S + 1e-6  is stated against.
 *
 * Rows are independent, so the loop over rows may run on several threads (OpenMP)
 * without changing any result bit.
 */
#include <stdint.h>
#include <math.h>
#include <string.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE 754 binary16 -> binary64, exact: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);              /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

/* Exported for the pin that checks the conversion against every one of the 65536 patterns. */
double oracle_half_to_double(uint16_t h) { return half_bits_to_double(h); }

/*
 * W: m x n FP16 bit patterns, row-major with leading dimension ld (>= n).
 * x: n FP16 bit patterns.  y, S: m doubles each (S may be NULL).
 * Returns the number of threads used.
 */
int oracle_spmv_f64(const uint16_t *W, int64_t m, int64_t n, int64_t ld,
                    const uint16_t *x, double *y, double *S)
{
    int threads = 1;
    /* The conversion is a pure function of 16 bits: tabulate it once (65536 doubles) and
       convert x once; the arithmetic below is unchanged. */
    double *tab = (double *)malloc(65536 * sizeof(double));
    double *xd = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    if (!tab || !xd) { free(tab); free(xd); return -1; }
    for (int h = 0; h < 65536; ++h) tab[h] = half_bits_to_double((uint16_t)h);
    for (int64_t j = 0; j < n; ++j) xd[j] = tab[x[j]];
#ifdef _OPENMP
    threads = omp_get_max_threads();
#pragma omp parallel for schedule(static)
#endif
    for (int64_t i = 0; i < m; ++i) {
        const uint16_t *row = W + i * ld;
        double acc = 0.0, mag = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            double p = tab[row[j]] * xd[j];
            acc += p;
            mag += fabs(p);
        }
        y[i] = acc;
        if (S) S[i] = mag;
    }
    free(tab);
    free(xd);
    return threads;
}

/*
 * The same definition for the paper's FP32 precision (Section 8 evaluates FP32 and FP16): W (m x n, leading dimension ld) and x are binary32; each input is converted exactly to FP64 (a C cast of a
 * float to double is exact), products and sums are FP64, columns in natural order.  y, S: m doubles each.
 * Returns the number of threads used.
 */
int oracle_spmv_f64_from_f32(const float *W, int64_t m, int64_t n, int64_t ld,
                             const float *x, double *y, double *S)
{
    int threads = 1;
#ifdef _OPENMP
    threads = omp_get_max_threads();
#pragma omp parallel for schedule(static)
#endif
    for (int64_t i = 0; i < m; ++i) {
        const float *row = W + i * ld;
        double acc = 0.0, mag = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            double p = (double)row[j] * (double)x[j];
            acc += p;
            mag += fabs(p);
        }
        y[i] = acc;
        if (S) S[i] = mag;
    }
    return threads;
}
