/* CPU oracle, integer GEMM step.  TEST INFRASTRUCTURE ONLY -- never linked into
 * or called by the product library.
 *
 * acc[m][c] = sum_j cx[m][j] * cw[c][j], the INT4 x INT4 product of the
 * quantised linear layer (paper: section "Methodology", quantised forward pass)
 * written as the plain triple loop in 64-bit integers.  Token rows are
 * independent, so the outer loop is shared among OpenMP threads; nothing else
 * is blocked, fused or reordered.
 *
 * cx [M][K], cw [N][K]: int8 codes in [-8, 7].  acc [M][N] int64.
 * Returns 0, or 1 if some accumulator does not fit a signed 32-bit integer
 * (the product path accumulates in int32).
 */
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int oracle_gemm_i4(const int8_t *cx, const int8_t *cw, int64_t M, int64_t N, int64_t K, int64_t *acc)
{
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t c = 0; c < N; ++c) {
            int64_t sum = 0;
            for (int64_t j = 0; j < K; ++j)
                sum += (int64_t)cx[m * K + j] * (int64_t)cw[c * K + j];
            acc[m * N + c] = sum;
            if (sum > INT32_MAX || sum < INT32_MIN)
                overflow = 1;
        }
    }
    return overflow;
}
