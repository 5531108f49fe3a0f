/*
 * CPU oracle for the NT / NN / transpose operations.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the ground truth the HIP kernels are checked against.  It is a
 * plain, slow, obviously-correct implementation and shares no code, header or
 * helper with the GPU path.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product never does.
 *
 * Every product is formed in double precision (the product of two floats is
 * exact in double) and accumulated in double in increasing order of the
 * summation index, so the result is the definition written out:
 *
 *   NN (Eq. 1):  C[i][j] = sum_l A[i][l] * B[l][j],  A m x k, B k x n
 *   NT (Eq. 2):  C[i][j] = sum_l A[i][l] * B[j][l],  A m x k, B n x k   (B^T_{ji} = B_{ij})
 *
 * with alpha = 1 and no beta*C term (Section II).  All matrices are row-major
 * with leading dimensions in elements.  Alongside C the routines return
 * S[i][j] = sum_l |A[i][l]| * |B..|, the denominator of the componentwise
 * rounding bound, so a test can state its tolerance relative to it.
 *
 * `rows`/`nrows` select which rows i of C are computed (NULL = all m rows);
 * the outputs then hold nrows x n values, row r belonging to C row rows[r].
 * Rows are independent, so they are spread over OpenMP threads; that is the
 * only parallelism and it does not change any sum.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. 2.  C and S may each be NULL. */
void oracle_nt_ref(int m, int n, int k,
                   const float *A, long lda, const float *B, long ldb,
                   const int *rows, int nrows,
                   double *C, double *S)
{
    int count = rows ? nrows : m;
    (void)m;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < count; ++r) {
        long i = rows ? rows[r] : r;
        for (long j = 0; j < n; ++j) {
            double acc = 0.0, mag = 0.0;
            for (long l = 0; l < k; ++l) {
                double a = (double)A[i * lda + l];
                double b = (double)B[j * ldb + l];
                acc += a * b;
                mag += fabs(a) * fabs(b);
            }
            if (C) C[(size_t)r * n + j] = acc;
            if (S) S[(size_t)r * n + j] = mag;
        }
    }
}

/* Eq. 1.  The l loop is outermost per row so that B is walked along its rows;
 * each C[i][j] still receives its terms in increasing l, one at a time. */
void oracle_nn_ref(int m, int n, int k,
                   const float *A, long lda, const float *B, long ldb,
                   const int *rows, int nrows,
                   double *C, double *S)
{
    int count = rows ? nrows : m;
    (void)m;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < count; ++r) {
        long i = rows ? rows[r] : r;
        double *acc = (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
        double *mag = (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
        for (long l = 0; l < k; ++l) {
            double a = (double)A[i * lda + l];
            for (long j = 0; j < n; ++j) {
                double b = (double)B[l * ldb + j];
                acc[j] += a * b;
                mag[j] += fabs(a) * fabs(b);
            }
        }
        for (long j = 0; j < n; ++j) {
            if (C) C[(size_t)r * n + j] = acc[j];
            if (S) S[(size_t)r * n + j] = mag[j];
        }
        free(acc);
        free(mag);
    }
}

/* Out-of-place transpose of 32-bit words: out[c][r] = in[r][c] (B^T_{ji} = B_{ij}).
 * Words are copied as integers so NaN payloads and signed zeros survive. */
void oracle_transpose_ref(int nrows, int ncols,
                          const uint32_t *in, long ldin, uint32_t *out, long ldout)
{
    for (long r = 0; r < nrows; ++r)
        for (long c = 0; c < ncols; ++c)
            out[c * ldout + r] = in[r * ldin + c];
}

/* The same two definitions on DOUBLE operands, for the training-step oracle (whose activations and
 * gradients are doubles, not floats): every C[i][j] is the definition's sum taken in increasing
 * order of the summation index, one term at a time.  All matrices dense row-major.
 *   nt:  C[i][j] = sum_l A[i][l] * B[j][l]     A m x k, B n x k   (Eq. 2: a layer's forward product)
 *   nn:  C[i][j] = sum_l A[i][l] * B[l][j]     A m x k, B k x n   (Eq. 1: the gradient w.r.t. a layer's input)
 *   tn:  C[i][j] = sum_r A[r][i] * B[r][j]     A k x m, B k x n   (Eq. 1 applied to A^T: the weight gradient,
 *                                                                  summed over the mini-batch index r) */
void oracle_f64_nt(int m, int n, int k, const double *A, const double *B, double *C)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < m; ++i)
        for (long j = 0; j < n; ++j) {
            double acc = 0.0;
            for (long l = 0; l < k; ++l) acc += A[(size_t)i * k + l] * B[(size_t)j * k + l];
            C[(size_t)i * n + j] = acc;
        }
}

void oracle_f64_nn(int m, int n, int k, const double *A, const double *B, double *C)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < m; ++i) {
        double *row = C + (size_t)i * n;
        for (long j = 0; j < n; ++j) row[j] = 0.0;
        for (long l = 0; l < k; ++l) {            /* element j of the row still gets its terms in increasing l */
            double a = A[(size_t)i * k + l];
            for (long j = 0; j < n; ++j) row[j] += a * B[(size_t)l * n + j];
        }
    }
}

void oracle_f64_tn(int m, int n, int k, const double *A, const double *B, double *C)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < m; ++i) {
        double *row = C + (size_t)i * n;
        for (long j = 0; j < n; ++j) row[j] = 0.0;
        for (long r = 0; r < k; ++r) {            /* ... in increasing r */
            double a = A[(size_t)r * m + i];
            for (long j = 0; j < n; ++j) row[j] += a * B[(size_t)r * n + j];
        }
    }
}
