/* Self-test of oracle/oracle.c built with the address and undefined-behaviour sanitizers:
 * exercises threads, leading dimensions, row subsets and the |a||b| output on small cases
 * whose results are known in closed form (identity, all-ones, rank one). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_sgemm_f64(int64_t batch, int64_t m, int64_t n, int64_t k, const float *A, int64_t lda, int64_t strideA,
                     const float *B, int64_t ldb, int64_t strideB, double *C, int64_t ldc, int64_t strideC, double *S,
                     const int64_t *rows, int64_t nrows, int threads);
int oracle_saxpy_f64(int64_t n, float alpha, const float *x, const float *y, double *z);

#define CHECK(cond)                                                                    \
    do {                                                                               \
        if (!(cond)) { fprintf(stderr, "oracle_selftest: failed: %s (line %d)\n", #cond, __LINE__); return 1; } \
    } while (0)

int main(void)
{
    enum { M = 7, N = 5, K = 9, LDA = 11, LDB = 6, BATCH = 3 };
    float *A = calloc((size_t)BATCH * M * LDA, sizeof(float));
    float *B = calloc((size_t)BATCH * K * LDB, sizeof(float));
    double *C = calloc((size_t)BATCH * M * N, sizeof(double));
    double *S = calloc((size_t)BATCH * M * N, sizeof(double));
    CHECK(A && B && C && S);
    /* rank one per problem: A[b][i][p] = i + 1 + b, B[b][p][j] = -(j + 1)  =>  C = -K (i+1+b)(j+1) */
    for (int b = 0; b < BATCH; ++b) {
        for (int i = 0; i < M; ++i) for (int p = 0; p < K; ++p) A[(b * M + i) * LDA + p] = (float)(i + 1 + b);
        for (int p = 0; p < K; ++p) for (int j = 0; j < N; ++j) B[(b * K + p) * LDB + j] = -(float)(j + 1);
    }
    for (int threads = 1; threads <= 40; threads += 13) {
        CHECK(oracle_sgemm_f64(BATCH, M, N, K, A, LDA, M * LDA, B, LDB, K * LDB, C, N, M * N, S, NULL, M, threads) == 0);
        for (int b = 0; b < BATCH; ++b) for (int i = 0; i < M; ++i) for (int j = 0; j < N; ++j) {
            CHECK(C[(b * M + i) * N + j] == -(double)K * (i + 1 + b) * (j + 1));
            CHECK(S[(b * M + i) * N + j] == (double)K * (i + 1 + b) * (j + 1));
        }
    }
    /* row subset, written compactly */
    int64_t rows[3] = {6, 0, 3};
    CHECK(oracle_sgemm_f64(BATCH, M, N, K, A, LDA, M * LDA, B, LDB, K * LDB, C, N, 3 * N, NULL, rows, 3, 4) == 0);
    for (int b = 0; b < BATCH; ++b) for (int s = 0; s < 3; ++s) for (int j = 0; j < N; ++j)
        CHECK(C[(b * 3 + s) * N + j] == -(double)K * (rows[s] + 1 + b) * (j + 1));
    /* argument errors */
    CHECK(oracle_sgemm_f64(1, M, N, K, A, K - 1, 0, B, LDB, 0, C, N, 0, NULL, NULL, M, 1) == 1);
    rows[0] = M;
    CHECK(oracle_sgemm_f64(1, M, N, K, A, LDA, 0, B, LDB, 0, C, N, 0, NULL, rows, 3, 1) == 1);
    CHECK(oracle_sgemm_f64(0, M, N, K, A, LDA, 0, B, LDB, 0, C, N, 0, NULL, NULL, M, 8) == 0);
    CHECK(oracle_sgemm_f64(1, M, N, 0, A, LDA, 0, B, LDB, 0, C, N, 0, NULL, NULL, M, 2) == 0 && C[0] == 0.0);
    /* axpy */
    float x[4] = {1, 2, 3, 4}, y[4] = {10, 20, 30, 40};
    double z[4];
    CHECK(oracle_saxpy_f64(4, -2.0f, x, y, z) == 0 && z[0] == 8 && z[3] == 32);
    CHECK(oracle_saxpy_f64(-1, 1.0f, x, y, z) == 1);
    free(A); free(B); free(C); free(S);
    printf("oracle_selftest: ok\n");
    return 0;
}
