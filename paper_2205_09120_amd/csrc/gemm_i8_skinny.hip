// int8 x int8 -> int32 GEMM for skinny right operands (N <= 16): the comparison point of gemm_i8_mfma for fully
// connected layers with a small batch, where a matrix-core tile would be almost empty.  The large operand A is
// streamed once from HBM; products are formed with packed 4 x int8 dot products (v_dot4_i32_i8).
//   * a workgroup (4 waves) owns 16 rows of A, a wave 4 rows; the 64 lanes split the depth, 16 bytes per lane and load;
//   * B is staged per depth chunk of 8192 into LDS, transposed to [column][depth] so that a lane reads the 16 depth
//     bytes matching its A bytes with one ds_read_b128 per column (8 columns per workgroup column block);
//   * each lane keeps 4 x 8 partial sums; a halving butterfly across lanes finishes the sums.
// HBM-bound: 1 byte of A per 2 lane-instructions.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

constexpr int NS8 = 8;       // columns per workgroup
constexpr int R8 = 4;        // rows per wave
constexpr int KC8 = 8192;    // depth bytes per LDS chunk (8 columns x 8 KiB = 64 KiB)
constexpr int J8 = KC8 / (64 * 16);

template <int CNT, int BIT> __device__ __forceinline__ void reduce_halving_i8(int32_t *val, int lane)
{
    if constexpr (BIT >= 1) {
        if constexpr (CNT > 1) {
            constexpr int HALF = CNT / 2;
            const bool upper = (lane & BIT) != 0;
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                const int32_t send = upper ? val[i] : val[i + HALF];
                const int32_t keep = upper ? val[i + HALF] : val[i];
                val[i] = keep + __shfl_xor(send, BIT, 64);
            }
            reduce_halving_i8<HALF, BIT / 2>(val, lane);
        } else {
            val[0] += __shfl_xor(val[0], BIT, 64);
            reduce_halving_i8<1, BIT / 2>(val, lane);
        }
    }
}

__device__ __forceinline__ int32_t dot4(uint32_t a, uint32_t b, int32_t c)
{
    return __builtin_amdgcn_sdot4((int)a, (int)b, c, false);
}

// FAST: A rows 16-byte aligned (lda % 16 == 0), B rows 8-byte aligned with ldb % 8 == 0
template <bool FAST>
__global__ __launch_bounds__(256) void gemm_i8_skinny_kernel(int M, int N, int K, const int8_t *__restrict__ A,
                                                             int64_t lda, const int8_t *__restrict__ B, int64_t ldb,
                                                             int32_t *__restrict__ C, int64_t ldc)
{
    __shared__ __attribute__((aligned(16))) uint32_t bt[NS8][KC8 / 4];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int m0 = (blockIdx.x * 4 + wave) * R8;
    const int n0 = blockIdx.y * NS8;

    int32_t acc[R8][NS8];
#pragma unroll
    for (int r = 0; r < R8; ++r)
#pragma unroll
        for (int n = 0; n < NS8; ++n)
            acc[r][n] = 0;

    // A: 16 bytes per lane and row; the loads of depth step j+1 are issued before step j is multiplied
    auto load_a = [&](uint4 (&a)[R8], int k0, bool whole) __attribute__((always_inline)) {
        const int k = k0 + lane * 16;
#pragma unroll
        for (int r = 0; r < R8; ++r) {
            const int row = m0 + r < M ? m0 + r : M - 1;
            const int8_t *src = A + (int64_t)row * lda;
            if (FAST && whole) {
                const uint32_t *p = reinterpret_cast<const uint32_t *>(src + k);
                a[r] = make_uint4(p[0], p[1], p[2], p[3]);
            } else {
                uint32_t w[4] = {0u, 0u, 0u, 0u};
                for (int i = 0; i < 16; ++i)
                    if (k + i < K)
                        w[i >> 2] |= (uint32_t)(uint8_t)src[k + i] << (8 * (i & 3));
                a[r] = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    };
    for (int kc = 0; kc < K; kc += KC8) {
        const bool whole = kc + KC8 <= K;  // uniform: the chunk lies inside the depth range
        uint4 a[R8], an[R8];
        load_a(a, kc, whole);
        if (kc)
            __syncthreads();
        // B chunk -> LDS, transposed: a thread takes 4 consecutive depth rows x 8 columns and writes one dword
        // (4 depth bytes) per column
#pragma unroll
        for (int u = tid; u < KC8 / 4; u += 256) {
            const int k = kc + u * 4;
            uint32_t lo[4], hi[4];  // per depth row: columns 0-3, columns 4-7
            if (FAST && n0 + NS8 <= N) {
                // straight-line loads from clamped addresses; rows past the depth are replaced by zero
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int kk = k + i < K ? k + i : K - 1;
                    const uint2 v = *reinterpret_cast<const uint2 *>(B + (int64_t)kk * ldb + n0);
                    lo[i] = k + i < K ? v.x : 0u;
                    hi[i] = k + i < K ? v.y : 0u;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    lo[i] = hi[i] = 0u;
                    if (k + i < K) {
                        const int8_t *src = B + (int64_t)(k + i) * ldb + n0;
                        for (int n = 0; n < NS8; ++n)
                            if (n0 + n < N) {
                                const uint32_t x = (uint32_t)(uint8_t)src[n] << (8 * (n & 3));
                                if (n < 4)
                                    lo[i] |= x;
                                else
                                    hi[i] |= x;
                            }
                    }
                }
            }
            // 4x4 byte transposes: column n gets its bytes from depth rows 0..3
            const uint32_t t0 = __builtin_amdgcn_perm(lo[1], lo[0], 0x05010400u), t1 = __builtin_amdgcn_perm(lo[1], lo[0], 0x07030602u);
            const uint32_t t2 = __builtin_amdgcn_perm(lo[3], lo[2], 0x05010400u), t3 = __builtin_amdgcn_perm(lo[3], lo[2], 0x07030602u);
            bt[0][u] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
            bt[1][u] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
            bt[2][u] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
            bt[3][u] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
            const uint32_t s0 = __builtin_amdgcn_perm(hi[1], hi[0], 0x05010400u), s1 = __builtin_amdgcn_perm(hi[1], hi[0], 0x07030602u);
            const uint32_t s2 = __builtin_amdgcn_perm(hi[3], hi[2], 0x05010400u), s3 = __builtin_amdgcn_perm(hi[3], hi[2], 0x07030602u);
            bt[4][u] = __builtin_amdgcn_perm(s2, s0, 0x05040100u);
            bt[5][u] = __builtin_amdgcn_perm(s2, s0, 0x07060302u);
            bt[6][u] = __builtin_amdgcn_perm(s3, s1, 0x05040100u);
            bt[7][u] = __builtin_amdgcn_perm(s3, s1, 0x07060302u);
        }
        __syncthreads();
        const int jmax = whole ? J8 : (K - kc + 1023) / 1024;
        for (int j = 0; j < jmax; ++j) {
            if (j + 1 < jmax)
                load_a(an, kc + (j + 1) * 1024, whole);
#pragma unroll
            for (int n = 0; n < NS8; ++n) {
                const uint4 b = *reinterpret_cast<const uint4 *>(&bt[n][(j * 64 + lane) * 4]);
#pragma unroll
                for (int r = 0; r < R8; ++r) {
                    int32_t s = acc[r][n];
                    s = dot4(a[r].x, b.x, s);
                    s = dot4(a[r].y, b.y, s);
                    s = dot4(a[r].z, b.z, s);
                    s = dot4(a[r].w, b.w, s);
                    acc[r][n] = s;
                }
            }
#pragma unroll
            for (int r = 0; r < R8; ++r)
                a[r] = an[r];
        }
    }

    int32_t val[R8 * NS8];
#pragma unroll
    for (int r = 0; r < R8; ++r)
#pragma unroll
        for (int n = 0; n < NS8; ++n)
            val[r * NS8 + n] = acc[r][n];
    reduce_halving_i8<R8 * NS8, 32>(val, lane);
    if ((lane & 1) == 0) {
        const int idx = lane >> 1;
        const int row = m0 + idx / NS8, col = n0 + idx % NS8;
        if (row < M && col < N)
            C[(int64_t)row * ldc + col] = val[0];
    }
}

}  // namespace

hipError_t launch_gemm_i8_skinny(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B,
                                 int64_t ldb, int32_t *C, int64_t ldc, hipStream_t stream)
{
    const int64_t gx = (M + 4 * R8 - 1) / (4 * R8), gy = (N + NS8 - 1) / NS8;
    if (gx > 0x7fffffffLL || gy > 65535)
        return hipErrorInvalidConfiguration;
    const bool fast = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 16 == 0) &&
                      (reinterpret_cast<uintptr_t>(B) % 8 == 0) && (ldb % 8 == 0);
    const dim3 g((unsigned)gx, (unsigned)gy), b(256);
    if (fast)
        hipLaunchKernelGGL(gemm_i8_skinny_kernel<true>, g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc);
    else
        hipLaunchKernelGGL(gemm_i8_skinny_kernel<false>, g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B, ldb, C,
                           ldc);
    return hipGetLastError();
}

}  // namespace lowbit
