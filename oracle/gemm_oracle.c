/*
 * CPU oracle for the low-bit GEMM (TEST INFRASTRUCTURE, not part of the product).
 *
 * The paper's binary / ternary / ternary-binary matrix multiplication is an exact
 * way of computing C = A B (Section II-A: A is m x k, B is k x n, C = AB; Section
 * III: the entries are restricted to {-1,+1} or {-1,0,+1}).  Because the method is
 * exact, the oracle is the definition itself, written out on the *unpacked* int8
 * values with 32-bit integer accumulation:
 *
 *     C[i][j] = sum_{t=0}^{k-1} A[i][t] * B[t][j]
 *
 * It never sees the packed representation and shares no code with the HIP kernels.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Loop order is i, t, j (row of A, depth, column of B).  Integer addition is
 * associative, so any order yields the same bits.
 */
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* A: M x K row-major (lda = K), B: K x N row-major (ldb = N), C: M x N row-major (ldc = N).
 * threads <= 0 means "whatever OpenMP picks".  Returns the number of threads used. */
int oracle_gemm_i8_i32(int64_t M, int64_t N, int64_t K, const int8_t *A, const int8_t *B, int32_t *C, int threads)
{
    int used = 1;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#else
    (void)threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        int32_t *c = C + i * N;
        memset(c, 0, (size_t)N * sizeof(int32_t));
        for (int64_t t = 0; t < K; ++t) {
            const int32_t a = (int32_t)A[i * K + t];
            const int8_t *b = B + t * N;
            for (int64_t j = 0; j < N; ++j)
                c[j] += a * (int32_t)b[j];
        }
    }
    return used;
}

/* Selected entries only: out[s] = sum_t A[ii[s]][t] * B[t][jj[s]].  Used to check
 * sampled outputs of problems whose full product is too slow to recompute. */
void oracle_gemm_i8_i32_samples(int64_t N, int64_t K, const int8_t *A, const int8_t *B, int64_t nsamples,
                                const int64_t *ii, const int64_t *jj, int32_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < nsamples; ++s) {
        const int8_t *a = A + ii[s] * K;
        const int8_t *b = B + jj[s];
        int32_t acc = 0;
        for (int64_t t = 0; t < K; ++t)
            acc += (int32_t)a[t] * (int32_t)b[t * N];
        out[s] = acc;
    }
}

/* 8-bit linear-quantized product with zero points, the left-hand side of eq. (3) of the paper written out:
 *     C[i][j] = sum_t (A[i][t] - zA) * (B[t][j] - zB)        A, B unsigned 8-bit, int32 accumulation. */
void oracle_gemm_u8_zp_i32(int64_t M, int64_t N, int64_t K, const uint8_t *A, const uint8_t *B, int32_t zA,
                           int32_t zB, int32_t *C)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        int32_t *c = C + i * N;
        memset(c, 0, (size_t)N * sizeof(int32_t));
        for (int64_t t = 0; t < K; ++t) {
            const int32_t a = (int32_t)A[i * K + t] - zA;
            const uint8_t *b = B + t * N;
            for (int64_t j = 0; j < N; ++j)
                c[j] += a * ((int32_t)b[j] - zB);
        }
    }
}
