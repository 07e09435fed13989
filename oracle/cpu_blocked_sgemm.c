/*
 * Blocked, multithreaded single-precision GEMM on the host CPU.  BASELINE ONLY (reported next
 * to the GPU numbers as context) and TEST INFRASTRUCTURE: nothing in the product path calls
 * it.  It computes the same operation as the oracle (first equation of the paper's
 * matrix-multiplication case study, C = alpha*op(A)*op(B) + beta*C, same `layout` bits) but in
 * fp32 with cache blocking: row panels of C are spread over threads (OpenMP), A and B blocks
 * are packed into contiguous buffers (which also absorbs the transposed storage), and the
 * innermost loop runs along a row of C so that the compiler vectorises it.
 * Checked against the oracle in tests/test_cpu_baseline.py.
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#define MC 64
#define KC 256
#define NC 1024

void cpu_blocked_sgemm(int M, int N, int K, float alpha, const float *A, int lda, const float *B,
                       int ldb, float beta, float *C, int ldc, int layout) {
    if (M <= 0 || N <= 0) return;
#pragma omp parallel
    {
        float *pa = (float *)malloc(sizeof(float) * MC * KC);
        float *pb = (float *)malloc(sizeof(float) * KC * NC);
        float *acc = (float *)malloc(sizeof(float) * MC * NC);
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int i0 = 0; i0 < M; i0 += MC) {
            for (int j0 = 0; j0 < N; j0 += NC) {
                const int mb = (M - i0 < MC) ? M - i0 : MC;
                const int nb = (N - j0 < NC) ? N - j0 : NC;
                memset(acc, 0, sizeof(float) * MC * NC);
                if (alpha != 0.0f) {
                    for (int k0 = 0; k0 < K; k0 += KC) {
                        const int kb = (K - k0 < KC) ? K - k0 : KC;
                        for (int i = 0; i < mb; ++i)
                            for (int k = 0; k < kb; ++k)
                                pa[i * KC + k] = (layout & 1) ? A[(size_t)(k0 + k) * lda + (i0 + i)]
                                                              : A[(size_t)(i0 + i) * lda + (k0 + k)];
                        for (int k = 0; k < kb; ++k)
                            for (int j = 0; j < nb; ++j)
                                pb[k * NC + j] = (layout & 2) ? B[(size_t)(j0 + j) * ldb + (k0 + k)]
                                                              : B[(size_t)(k0 + k) * ldb + (j0 + j)];
                        for (int i = 0; i < mb; ++i) {
                            float *restrict row = acc + (size_t)i * NC;
                            for (int k = 0; k < kb; ++k) {
                                const float a = pa[i * KC + k];
                                const float *restrict brow = pb + (size_t)k * NC;
                                for (int j = 0; j < nb; ++j) row[j] += a * brow[j];
                            }
                        }
                    }
                }
                for (int i = 0; i < mb; ++i) {
                    float *c = C + (size_t)(i0 + i) * ldc + j0;
                    const float *row = acc + (size_t)i * NC;
                    if (beta == 0.0f)
                        for (int j = 0; j < nb; ++j) c[j] = alpha * row[j];
                    else
                        for (int j = 0; j < nb; ++j) c[j] = alpha * row[j] + beta * c[j];
                }
            }
        }
        free(pa);
        free(pb);
        free(acc);
    }
}

#ifdef _OPENMP
#include <omp.h>
int cpu_blocked_threads(void) { return omp_get_max_threads(); }
#else
int cpu_blocked_threads(void) { return 1; }
#endif
