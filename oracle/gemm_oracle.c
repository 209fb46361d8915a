/*
 * CPU oracle for the matrix product.  TEST INFRASTRUCTURE ONLY (tests, smoke check, the
 * benchmark's CPU-baseline leg); the library never calls it.
 *
 * It is the paper's three-loop matrix multiplication (figure "Matrix multiplication code",
 * section "Notation"): C[i][j] += A[i][k] * B[k][j], all matrices row-major, A is M x K,
 * B is K x N, C is M x N.  The GEMM section writes C = beta*C + alpha*A*B; the reading taken
 * is alpha = beta = 1 by default (the baseline listing there applies beta inside the k loop,
 * which only makes sense for beta = 1), and general alpha, beta are applied once per element:
 * C = beta*C0 + alpha * sum_k A[i][k]*B[k][j].
 *
 * Every product and sum is IEEE double, k ascending.  absum = |beta*C0| + |alpha| * sum |a*b|.
 *
 * Pinned by tests/test_oracle_gemm.py: B = identity, A = ones (column sums), a 2x2 worked by
 * hand, exact integer products against numpy int64, and the conv oracle on 1x1 filters.
 */
#include <stdint.h>
#include <math.h>

static void gemm_point(int64_t N, int64_t K, const float *A, const float *B, const float *C0,
                       double alpha, double beta, int64_t i, int64_t j, double *y, double *scale)
{
    double acc = 0.0, mag = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        double a = (double)A[i * K + k];
        double b = (double)B[k * N + j];
        acc += a * b;
        mag += fabs(a * b);
    }
    double c0 = C0 ? beta * (double)C0[i * N + j] : 0.0;
    *y = c0 + alpha * acc;
    *scale = fabs(c0) + fabs(alpha) * mag;
}

int oracle_gemm(int64_t M, int64_t N, int64_t K, const float *A, const float *B, const float *C0,
                double alpha, double beta, double *C, double *absum)
{
    if (M <= 0 || N <= 0 || K < 0)
        return -1;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j)
            gemm_point(N, K, A, B, C0, alpha, beta, i, j, &C[i * N + j], &absum[i * N + j]);
    return 0;
}

/* Only the elements whose flat row-major indices are listed in idx[0..count). */
int oracle_gemm_at(int64_t M, int64_t N, int64_t K, const float *A, const float *B, const float *C0,
                   double alpha, double beta, int64_t count, const int64_t *idx,
                   double *C, double *absum)
{
    if (M <= 0 || N <= 0 || K < 0)
        return -1;
    for (int64_t t = 0; t < count; ++t)
        if (idx[t] < 0 || idx[t] >= M * N)
            return -2;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t)
        gemm_point(N, K, A, B, C0, alpha, beta, idx[t] / N, idx[t] % N, &C[t], &absum[t]);
    return 0;
}
