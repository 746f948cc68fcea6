/* CPU oracle, integer contraction only.  TEST INFRASTRUCTURE: linked by the
 * tests, the smoke check and the benchmark's cpu_baseline leg, never by the
 * product path.  Shares no code with the HIP kernels.
 *
 * acc[m][n] = sum_k q[m][k] * w[n][k]
 * is the definition of the quantized linear layer's integer product (paper
 * Section 4.4: one layer-wise activation grid, 4-bit weights, wide
 * accumulation).  Plain loops in the order m, n, k; a 64-bit running sum is
 * checked against the 32-bit accumulator the method uses.
 *
 * q : int8 [M][K] codes of Eq.2 on the signed grid (zero-point 0)
 * w : int8 [N][K] with values in [-8, 7]
 * Returns 0, or 1 if some accumulator leaves int32 (output then undefined).
 * `threads` > 1 splits the rows m over OpenMP threads. */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int agq_oracle_gemm_i8(const int8_t *q, const int8_t *w, int64_t M,
                       int64_t N, int64_t K, int32_t *acc, int threads)
{
    int bad = 0;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static) reduction(| : bad)
#endif
    for (int64_t m = 0; m < M; ++m) {
        const int8_t *qr = q + m * K;
        for (int64_t n = 0; n < N; ++n) {
            const int8_t *wr = w + n * K;
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)((int32_t)qr[k] * (int32_t)wr[k]);
            if (s > INT32_MAX || s < INT32_MIN) bad = 1;
            acc[m * N + n] = (int32_t)s;
        }
    }
    return bad;
}

int agq_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
