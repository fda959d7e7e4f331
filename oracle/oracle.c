/*
 * CPU oracle for dense matrix multiplication -- TEST INFRASTRUCTURE ONLY.
 *
 * Computes the definition of "matmul" in Sec. 5.2 of the paper: C = A.B with A of
 * size m x k and B of size k x n, i.e. C[i][j] = sum_{p=0}^{k-1} A[i][p] * B[p][j],
 * written out as the plain triple loop.  The batched form applies the same
 * definition independently to every problem of the batch.
 *
 * Precision: every fp32 input is widened to fp64; the product of two fp32 values is
 * exact in fp64; the running sum is fp64 and adds the terms in ascending p.  For
 * k <= 2^24 the result differs from the exact sum by at most k * 2^-53 * sum|a||b|.
 *
 * Layout: row-major with leading dimensions (A[i*lda+p], B[p*ldb+j], C[i*ldc+j]);
 * problem b of a batch starts at A + b*strideA, B + b*strideB, C + b*strideC.
 * The paper's matrices are column-major; a column-major product is the row-major
 * product of the swapped operands, so this one routine covers both.
 *
 * Loop order is i, p, j with an n-long fp64 row of running sums, so each C[i][j]
 * still receives its k terms in ascending p.  Rows are divided statically between
 * host threads; no element's arithmetic depends on the thread count.
 *
 * This file shares nothing with the GPU library: no headers, helpers or constants.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * Pinned by tests/test_oracle_pins.py (identity, all-ones, exact-rational brute
 * force, closed forms, transpose/K-additivity invariants, Freivalds, dgemm).
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>

typedef struct {
    int64_t m, n, k;
    const float *A; int64_t lda, strideA;
    const float *B; int64_t ldb, strideB;
    double *C;      int64_t ldc, strideC;
    double *S;      /* optional: sum_p |A[i][p]| * |B[p][j]|, same layout as C; may be NULL */
    const int64_t *rows; /* optional list of row indices (NULL = all rows 0..m-1) */
    int64_t nrows;       /* number of rows computed per problem */
    int64_t unit_begin, unit_end; /* range of (problem, row-slot) units for this thread */
} job_t;

/* One output row: out[j] = sum_p a[p] * B[p][j]; optionally sabs[j] = sum_p |a[p]| |B[p][j]|. */
static void one_row(const float *a, const float *B, int64_t ldb, int64_t n, int64_t k,
                    double *out, double *sabs)
{
    for (int64_t j = 0; j < n; ++j) out[j] = 0.0;
    if (sabs) for (int64_t j = 0; j < n; ++j) sabs[j] = 0.0;
    for (int64_t p = 0; p < k; ++p) {
        const double aip = (double)a[p];
        const float *brow = B + p * ldb;
        for (int64_t j = 0; j < n; ++j) out[j] += aip * (double)brow[j];
        if (sabs) {
            const double aabs = fabs(aip);
            for (int64_t j = 0; j < n; ++j) sabs[j] += aabs * fabs((double)brow[j]);
        }
    }
}

static void *worker(void *arg)
{
    const job_t *jb = (const job_t *)arg;
    for (int64_t u = jb->unit_begin; u < jb->unit_end; ++u) {
        const int64_t b = u / jb->nrows;
        const int64_t slot = u % jb->nrows;
        const int64_t i = jb->rows ? jb->rows[slot] : slot;
        const float *a = jb->A + b * jb->strideA + i * jb->lda;
        const float *B = jb->B + b * jb->strideB;
        double *out = jb->C + b * jb->strideC + slot * jb->ldc;
        double *sabs = jb->S ? jb->S + b * jb->strideC + slot * jb->ldc : NULL;
        one_row(a, B, jb->ldb, jb->n, jb->k, out, sabs);
    }
    return NULL;
}

/*
 * Batched row-major GEMM in fp64.  If rows != NULL only the nrows listed rows of each
 * problem are computed and written compactly: output row slot s (0 <= s < nrows) holds
 * C[rows[s]][*]; C then needs nrows*ldc doubles per problem.  With rows == NULL pass
 * nrows = m.  S may be NULL.  threads <= 0 selects one thread.
 * Returns 0 on success, 1 on an invalid argument, 2 if host memory ran out.
 */
int oracle_sgemm_f64(int64_t batch, int64_t m, int64_t n, int64_t k,
                     const float *A, int64_t lda, int64_t strideA,
                     const float *B, int64_t ldb, int64_t strideB,
                     double *C, int64_t ldc, int64_t strideC, double *S,
                     const int64_t *rows, int64_t nrows, int threads)
{
    if (batch < 0 || m < 0 || n < 0 || k < 0 || nrows < 0) return 1;
    if (lda < k || ldb < n || ldc < n) return 1;
    if (!rows && nrows != m) return 1;
    if (rows) for (int64_t s = 0; s < nrows; ++s) if (rows[s] < 0 || rows[s] >= m) return 1;
    const int64_t units = batch * nrows;
    if (units == 0 || n == 0) return 0;
    if (threads < 1) threads = 1;
    if ((int64_t)threads > units) threads = (int)units;

    job_t *jobs = (job_t *)calloc((size_t)threads, sizeof(job_t));
    pthread_t *tids = (pthread_t *)calloc((size_t)threads, sizeof(pthread_t));
    char *joinable = (char *)calloc((size_t)threads, 1);
    if (!jobs || !tids || !joinable) { free(jobs); free(tids); free(joinable); return 2; }
    for (int t = 0; t < threads; ++t) {
        job_t *jb = &jobs[t];
        jb->m = m; jb->n = n; jb->k = k;
        jb->A = A; jb->lda = lda; jb->strideA = strideA;
        jb->B = B; jb->ldb = ldb; jb->strideB = strideB;
        jb->C = C; jb->ldc = ldc; jb->strideC = strideC; jb->S = S;
        jb->rows = rows; jb->nrows = nrows;
        jb->unit_begin = units * t / threads;
        jb->unit_end = units * (t + 1) / threads;
        /* The last share runs on the calling thread; so does any share whose thread
         * cannot be created, so the result is complete either way. */
        if (t == threads - 1 || pthread_create(&tids[t], NULL, worker, jb) != 0) worker(jb);
        else joinable[t] = 1;
    }
    for (int t = 0; t < threads; ++t) if (joinable[t]) pthread_join(tids[t], NULL);
    free(jobs); free(tids); free(joinable);
    return 0;
}

/*
 * axpy of Sec. 5.2 of the paper: z = alpha.x + y on vectors of n elements, written as the
 * definition.  alpha and x[i] are fp32, their product is exact in fp64; the sum with y[i] is
 * one fp64 addition (relative error <= 2^-53).  Returns 0, or 1 on an invalid argument.
 */
int oracle_saxpy_f64(int64_t n, float alpha, const float *x, const float *y, double *z)
{
    if (n < 0) return 1;
    for (int64_t i = 0; i < n; ++i) z[i] = (double)alpha * (double)x[i] + (double)y[i];
    return 0;
}

/* Number of online host cores (used as the default thread count by the Python side). */
int oracle_host_cores(void)
{
    long c = sysconf(_SC_NPROCESSORS_ONLN);
    return c > 0 ? (int)c : 1;
}
