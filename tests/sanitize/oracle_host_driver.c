/* Runs every function of the C oracle (oracle/gemm_oracle.c, compiled into this program with AddressSanitizer and
 * UndefinedBehaviorSanitizer) on operands held in heap blocks of exactly their size, at the extreme values of each
 * type, and checks the results against sums that have a closed form.  A read or write past an operand, or a signed
 * overflow in the accumulation, ends the program with a sanitizer report.  tests/test_sanitizers.py builds and runs it. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_gemm_i8_i32(int64_t M, int64_t N, int64_t K, const int8_t *A, const int8_t *B, int32_t *C, int threads);
void oracle_gemm_i8_i32_samples(int64_t N, int64_t K, const int8_t *A, const int8_t *B, int64_t nsamples,
                                const int64_t *ii, const int64_t *jj, int32_t *out);
void oracle_gemm_u8_zp_i32(int64_t M, int64_t N, int64_t K, const uint8_t *A, const uint8_t *B, int32_t zA, int32_t zB,
                           int32_t *C);

static int failures = 0;
#define EXPECT(c)                                                \
    do {                                                         \
        if (!(c)) {                                              \
            printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); \
            ++failures;                                          \
        }                                                        \
    } while (0)

static uint32_t lcg(uint32_t *s) { return *s = *s * 1664525u + 1013904223u; }

static void constant_operands(int64_t M, int64_t N, int64_t K, int a, int b)
{
    int8_t *A = malloc((size_t)(M * K)), *B = malloc((size_t)(K * N));
    int32_t *C = malloc((size_t)(M * N) * sizeof(int32_t));
    memset(A, a, (size_t)(M * K));
    memset(B, b, (size_t)(K * N));
    const int used = oracle_gemm_i8_i32(M, N, K, A, B, C, 3);
    EXPECT(used >= 1);
    for (int64_t x = 0; x < M * N; ++x)
        EXPECT(C[x] == (int32_t)(K * (int64_t)(int8_t)a * (int8_t)b));
    free(A), free(B), free(C);
}

static void random_against_samples(int64_t M, int64_t N, int64_t K, int ternary)
{
    uint32_t s = (uint32_t)(M * 7919 + N * 104729 + K);
    int8_t *A = malloc((size_t)(M * K)), *B = malloc((size_t)(K * N));
    int32_t *C = malloc((size_t)(M * N) * sizeof(int32_t));
    for (int64_t x = 0; x < M * K; ++x)
        A[x] = ternary ? (int8_t)((lcg(&s) >> 16) % 3) - 1 : (int8_t)(lcg(&s) >> 24);
    for (int64_t x = 0; x < K * N; ++x)
        B[x] = ternary ? (int8_t)((lcg(&s) >> 16) % 3) - 1 : (int8_t)(lcg(&s) >> 24);
    oracle_gemm_i8_i32(M, N, K, A, B, C, 0);
    /* every entry again through the sampled-entries routine, indices in blocks of exactly their size */
    const int64_t n = M * N;
    int64_t *ii = malloc((size_t)n * sizeof(int64_t)), *jj = malloc((size_t)n * sizeof(int64_t));
    int32_t *out = malloc((size_t)n * sizeof(int32_t));
    for (int64_t x = 0; x < n; ++x)
        ii[x] = x / N, jj[x] = x % N;
    oracle_gemm_i8_i32_samples(N, K, A, B, n, ii, jj, out);
    EXPECT(memcmp(out, C, (size_t)n * sizeof(int32_t)) == 0);
    /* and one entry by the definition, written out here */
    int64_t acc = 0;
    for (int64_t t = 0; t < K; ++t)
        acc += (int64_t)A[(M - 1) * K + t] * B[t * N + (N - 1)];
    EXPECT(C[n - 1] == (int32_t)acc);
    free(A), free(B), free(C), free(ii), free(jj), free(out);
}

static void zero_point_product(int64_t M, int64_t N, int64_t K, int a, int b, int zA, int zB)
{
    uint8_t *A = malloc((size_t)(M * K)), *B = malloc((size_t)(K * N));
    int32_t *C = malloc((size_t)(M * N) * sizeof(int32_t));
    memset(A, a, (size_t)(M * K));
    memset(B, b, (size_t)(K * N));
    oracle_gemm_u8_zp_i32(M, N, K, A, B, zA, zB, C);
    for (int64_t x = 0; x < M * N; ++x)
        EXPECT(C[x] == (int32_t)(K * (int64_t)(a - zA) * (b - zB)));
    free(A), free(B), free(C);
}

/* Shows that the instrumentation is live: a right operand one byte short must end in a sanitizer report. */
static int lie_about_an_operand(void)
{
    int8_t *A = malloc(4 * 8), *B = malloc(8 * 4 - 1);
    int32_t *C = malloc(4 * 4 * sizeof(int32_t));
    memset(A, 1, 4 * 8);
    memset(B, 1, 8 * 4 - 1);
    oracle_gemm_i8_i32(4, 4, 8, A, B, C, 1);
    printf("the short operand went unnoticed\n");
    return 0;
}

int main(int argc, char **argv)
{
    if (argc > 1 && strcmp(argv[1], "--lie") == 0)
        return lie_about_an_operand();
    /* extreme values: (-128)^2 * K stays below 2^31 for K <= 131071, the depth limit of the 8-bit comparator */
    constant_operands(3, 5, 131071, -128, -128);
    constant_operands(2, 2, 131071, -128, 127);
    constant_operands(7, 1, 1, 127, 127);
    constant_operands(1, 9, 64, -1, 1);
    constant_operands(1, 1, 32767, 1, -1); /* k_max of Table II */
    /* empty extents: nothing is touched (zero-size blocks) */
    constant_operands(0, 4, 16, 1, 1);
    constant_operands(4, 0, 16, 1, 1);
    random_against_samples(17, 33, 129, 1);
    random_against_samples(5, 3, 1000, 0);
    random_against_samples(1, 1, 1, 1);
    random_against_samples(64, 65, 63, 1);
    zero_point_product(3, 4, 33025, 255, 255, 0, 0);  /* 255^2 * 33025 < 2^31 */
    zero_point_product(3, 4, 33025, 0, 0, 255, 255);
    zero_point_product(2, 2, 1000, 0, 255, 255, 0);   /* negative products */
    zero_point_product(0, 2, 10, 1, 1, 1, 1);
    printf(failures ? "%d expectation(s) failed\n" : "all expectations hold (%d failures)\n", failures);
    return failures != 0;
}
