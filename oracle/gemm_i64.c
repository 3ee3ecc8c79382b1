/* CPU oracle, integer GEMM (TEST INFRASTRUCTURE ONLY; never linked into the product).
 *
 * acc[m][n] = sum_k qx[m][k] * w[n][k], every product and the sum in int64
 * (the INT8 matrix multiplication of Section 4.1 of arXiv 2405.04532, "as if it was
 * W8A8 per-channel").  Plain triple loop in the order of the definition; the only
 * parallelism is OpenMP over output rows.  No blocking, no intrinsics.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC gemm_i64.c -o libqoq_oracle.so
 */
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* qx: [M][K] int8 row-major; w: [N][K] int8 row-major; acc: [M][N] int64. */
void oracle_gemm_i8_i64(const int8_t* qx, const int8_t* w, int64_t* acc,
                        int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t mn = 0; mn < M * N; ++mn) {
        const int64_t m = mn / N, n = mn % N;
        const int8_t* a = qx + m * K;
        const int8_t* b = w + n * K;
        int64_t s = 0;
        for (int64_t k = 0; k < K; ++k)
            s += (int64_t)a[k] * (int64_t)b[k];
        acc[m * N + n] = s;
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
