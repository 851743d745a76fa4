// int8 x int8 -> int32 GEMM on the gfx950 integer matrix cores (v_mfma_i32_32x32x32_i8).
//
// Comparison point for the popcount kernels: it computes the same C = A B from unpacked int8 operands, the role
// the 8-bit gemmlowp multiplication (U8) plays in Section IV of the paper.
//
// Workgroup tile 128 x 128, depth step 64, 4 waves in a 2 x 2 arrangement, each wave 64 x 64 = 2 x 2 MFMA tiles.
//   A (row-major, depth contiguous) is staged as is:   As[row][64 depth bytes (+16 pad)].
//   B (row-major, depth strided) is transposed on the way: a thread loads 4 depth rows x 4 columns (4 dwords),
//   transposes the 4x4 bytes in registers and stores, per column, one dword holding 4 consecutive depth bytes:
//   Bs[depth/4][column] (dwords).
// Both MFMA operands take 16 depth bytes per lane (lane%32 = row / column, lane/32 = which half of the 32 deep
// step); A and B use the same slot order, so the order of depth positions inside the instruction does not matter.
// The next depth step is fetched into registers while the current one is multiplied.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int A_STRIDE = BK + 16;     // bytes per staged A row
constexpr int B_STRIDE = BN + 4;      // dwords per staged B depth-quad row

__device__ __forceinline__ uint32_t load_a_bytes(const int8_t *p, int n)
{
    uint32_t x = 0;
    for (int i = 0; i < n; ++i)
        x |= (uint32_t)(uint8_t)p[i] << (8 * i);
    return x;
}

template <bool FAST>
__global__ __launch_bounds__(256) void gemm_i8_mfma_kernel(int M, int N, int K, const int8_t *__restrict__ A,
                                                           int64_t lda, const int8_t *__restrict__ B, int64_t ldb,
                                                           int32_t *__restrict__ C, int64_t ldc, int nMB, int nNB,
                                                           int tiles_per_xcd)
{
    __shared__ __attribute__((aligned(16))) uint8_t As[BM * A_STRIDE];
    __shared__ __attribute__((aligned(16))) uint32_t Bs[(BK / 4) * B_STRIDE];

    const int bid = blockIdx.x;
    const int idx = (bid & 7) * tiles_per_xcd + (bid >> 3);
    if ((bid >> 3) >= tiles_per_xcd || idx >= nMB * nNB)
        return;
    const int nb = idx / nMB, mb = idx - nb * nMB;   // M blocks of one N block are adjacent (share the B tile)
    const int m0 = mb * BM, n0 = nb * BN;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave & 1, wn = wave >> 1;

    // staging assignments
    const int a_row = tid >> 2, a_col = (tid & 3) * 16;          // + 64 rows on the second pass
    const int b_nq = tid & 31, b_kq = tid >> 5;                  // + 8 depth quads on the second pass

    uint4 a_pre[2];
    uint32_t b_pre[2][4];

    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int r = m0 + a_row + p * 64, k = k0 + a_col;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (r < M && k < K) {
                const int8_t *src = A + (int64_t)r * lda + k;
                if (FAST && k + 16 <= K) {
                    v = *reinterpret_cast<const uint4 *>(src);
                } else {
                    const int n = (K - k) < 16 ? (K - k) : 16;
                    v.x = load_a_bytes(src, n < 4 ? n : 4);
                    v.y = n > 4 ? load_a_bytes(src + 4, (n - 4) < 4 ? (n - 4) : 4) : 0u;
                    v.z = n > 8 ? load_a_bytes(src + 8, (n - 8) < 4 ? (n - 8) : 4) : 0u;
                    v.w = n > 12 ? load_a_bytes(src + 12, (n - 12) < 4 ? (n - 12) : 4) : 0u;
                }
            }
            a_pre[p] = v;
        }
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int n = n0 + b_nq * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k = k0 + (b_kq + p * 8) * 4 + j;
                uint32_t x = 0u;
                if (k < K && n < N) {
                    const int8_t *src = B + (int64_t)k * ldb + n;
                    if (FAST && n + 4 <= N)
                        x = *reinterpret_cast<const uint32_t *>(src);
                    else
                        x = load_a_bytes(src, (N - n) < 4 ? (N - n) : 4);
                }
                b_pre[p][j] = x;
            }
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int p = 0; p < 2; ++p)
            *reinterpret_cast<uint4 *>(&As[(a_row + p * 64) * A_STRIDE + a_col]) = a_pre[p];
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            // rows = depth j, bytes = column i  ->  out[i] byte j = in[j] byte i
            const uint32_t r0 = b_pre[p][0], r1 = b_pre[p][1], r2 = b_pre[p][2], r3 = b_pre[p][3];
            const uint32_t t0 = __builtin_amdgcn_perm(r1, r0, 0x05010400u);  // r0.b0 r1.b0 r0.b1 r1.b1
            const uint32_t t1 = __builtin_amdgcn_perm(r1, r0, 0x07030602u);  // r0.b2 r1.b2 r0.b3 r1.b3
            const uint32_t t2 = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
            const uint32_t t3 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
            uint4 o;
            o.x = __builtin_amdgcn_perm(t2, t0, 0x05040100u);  // col0: r0.b0 r1.b0 r2.b0 r3.b0
            o.y = __builtin_amdgcn_perm(t2, t0, 0x07060302u);  // col1
            o.z = __builtin_amdgcn_perm(t3, t1, 0x05040100u);  // col2
            o.w = __builtin_amdgcn_perm(t3, t1, 0x07060302u);  // col3
            *reinterpret_cast<uint4 *>(&Bs[(b_kq + p * 8) * B_STRIDE + b_nq * 4]) = o;
        }
    };

    v16i acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    const int nsteps = (K + BK - 1) / BK;
    fetch(0);
    for (int s = 0; s < nsteps; ++s) {
        commit();
        __syncthreads();
        if (s + 1 < nsteps)
            fetch((s + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = wm * 64 + i * 32 + (lane & 31);
                af[i] = *reinterpret_cast<const v4i *>(&As[row * A_STRIDE + ks * 32 + (lane >> 5) * 16]);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = wn * 64 + j * 32 + (lane & 31);
                const int kq = ks * 8 + (lane >> 5) * 4;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    bf[j][q] = (int)Bs[(kq + q) * B_STRIDE + col];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator layout of the 32x32 tile: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < M && col < N)
                    C[(int64_t)row * ldc + col] = acc[i][j][r];
            }
        }
}

}  // namespace

hipError_t launch_gemm_i8(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                          int32_t *C, int64_t ldc, hipStream_t stream)
{
    const int nMB = (int)((M + BM - 1) / BM), nNB = (int)((N + BN - 1) / BN);
    const int64_t tiles = (int64_t)nMB * nNB;
    const int tiles_per_xcd = (int)((tiles + 7) / 8);
    const int64_t grid = (int64_t)tiles_per_xcd * 8;
    if (grid > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    const bool fast = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 16 == 0) &&
                      (reinterpret_cast<uintptr_t>(B) % 4 == 0) && (ldb % 4 == 0);
    if (fast)
        hipLaunchKernelGGL(gemm_i8_mfma_kernel<true>, dim3((unsigned)grid), dim3(256), 0, stream, (int)M, (int)N,
                           (int)K, A, lda, B, ldb, C, ldc, nMB, nNB, tiles_per_xcd);
    else
        hipLaunchKernelGGL(gemm_i8_mfma_kernel<false>, dim3((unsigned)grid), dim3(256), 0, stream, (int)M, (int)N,
                           (int)K, A, lda, B, ldb, C, ldc, nMB, nNB, tiles_per_xcd);
    return hipGetLastError();
}

}  // namespace lowbit
