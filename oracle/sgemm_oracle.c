/*
 * CPU oracle for single-precision GEMM.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product path may call, link or import this file; it shares no code with the GPU
 * library.
 *
 * What it computes is the plain definition of the operation in the paper's
 * matrix-multiplication case study (section "Case-study: matrix-multiplication",
 * first equation):  C = alpha * op(A) * B' + beta * C,  i.e. for every 0<=i<M, 0<=j<N
 *
 *     C_out[i][j] = alpha * sum_{k=0}^{K-1} A(i,k) * B(k,j)  +  beta * C_in[i][j]
 *
 * The paper stores A transposed (its "A^T B" form); here bit 0 of `layout` selects
 * that storage, bit 1 does the same for B:
 *     A(i,k) = A[i*lda + k]   (layout bit 0 clear, A stored M x K row-major)
 *            = A[k*lda + i]   (layout bit 0 set,   A stored K x M row-major)
 *     B(k,j) = B[k*ldb + j]   (layout bit 1 clear, B stored K x N row-major)
 *            = B[j*ldb + k]   (layout bit 1 set,   B stored N x K row-major)
 * C_in is M x N row-major with leading dimension ldc; C_out is dense M x N doubles.
 *
 * Arithmetic: every product is formed in double from the two floats (exact: 24+24
 * significand bits fit in 53), the sum runs in double in increasing k, and
 * (double)alpha*sum + (double)beta*(double)C_in is evaluated in double.
 *
 * Readings where the paper is silent (BLAS convention):
 *   beta == 0  : C_in is never read, so NaN/Inf there cannot reach the result.
 *   alpha == 0 : A and B are never read; the sum term is exactly 0.
 *   K == 0     : the sum is empty (0).
 *
 * Parity pins (tests/test_oracle_sgemm.py): identity and permutation matrices,
 * closed-form rank-1 sums, alpha/beta edge cases, brute force on tiny integer
 * inputs with an independent pure-Python loop, layout identities, and agreement
 * with numpy's fp64 matmul.
 *
 * Rows are independent, so the outer loop may run on several threads (OpenMP)
 * without changing any value.
 */
#include <stddef.h>

static double a_at(const float *A, int lda, int layout, int i, int k) {
    return (layout & 1) ? (double)A[(size_t)k * (size_t)lda + (size_t)i]
                        : (double)A[(size_t)i * (size_t)lda + (size_t)k];
}

static double b_at(const float *B, int ldb, int layout, int k, int j) {
    return (layout & 2) ? (double)B[(size_t)j * (size_t)ldb + (size_t)k]
                        : (double)B[(size_t)k * (size_t)ldb + (size_t)j];
}

/* One element of the result, straight from the definition. */
static double element(int K, float alpha, const float *A, int lda, const float *B, int ldb,
                      float beta, const float *C_in, int ldc, int layout, int i, int j) {
    double sum = 0.0;
    if (alpha != 0.0f) {
        for (int k = 0; k < K; ++k) {
            sum += a_at(A, lda, layout, i, k) * b_at(B, ldb, layout, k, j);
        }
    }
    double r = (double)alpha * sum;
    if (beta != 0.0f) {
        r += (double)beta * (double)C_in[(size_t)i * (size_t)ldc + (size_t)j];
    }
    return r;
}

/* Full result: C_out is dense M x N (row-major, leading dimension N), doubles. */
void oracle_sgemm(int M, int N, int K, float alpha, const float *A, int lda, const float *B,
                  int ldb, float beta, const float *C_in, int ldc, int layout, double *C_out) {
#pragma omp parallel for schedule(dynamic, 4)
    for (int i = 0; i < M; ++i) {
        for (int j = 0; j < N; ++j) {
            C_out[(size_t)i * (size_t)N + (size_t)j] =
                element(K, alpha, A, lda, B, ldb, beta, C_in, ldc, layout, i, j);
        }
    }
}

/* Sampled result: out[s] = C_out[rows[s]][cols[s]] for s in [0, count).  Every element is
 * an independent dot product, so these are exact oracle values at any problem size. */
void oracle_sgemm_sample(int M, int N, int K, float alpha, const float *A, int lda,
                         const float *B, int ldb, float beta, const float *C_in, int ldc,
                         int layout, long long count, const int *rows, const int *cols,
                         double *out) {
    (void)M;
    (void)N;
#pragma omp parallel for schedule(dynamic, 64)
    for (long long s = 0; s < count; ++s) {
        out[s] = element(K, alpha, A, lda, B, ldb, beta, C_in, ldc, layout, rows[s], cols[s]);
    }
}

/* Number of threads the loops above use (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int oracle_threads(void) { return omp_get_max_threads(); }
#else
int oracle_threads(void) { return 1; }
#endif
