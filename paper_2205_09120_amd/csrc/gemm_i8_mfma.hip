// int8 x int8 -> int32 GEMM on the gfx950 integer matrix cores (v_mfma_i32_32x32x32_i8).
//
// Comparison point for the popcount kernels: it computes the same C = A B from unpacked int8 operands, the role
// the 8-bit gemmlowp multiplication (U8) plays in Section IV of the paper.
//
// Workgroup = 4 waves in a 2 x 2 arrangement; a wave computes TM x TN MFMA tiles of 32 x 32, so the workgroup
// tile is (64*TM) x (64*TN); depth step 64 (two MFMA depth steps of 32).  Instances: 256 x 128 (TM=4, TN=2)
// for large problems, 128 x 128 (TM=TN=2) for small ones, 256 x 256 selectable for experiments.
//   A (row-major, depth contiguous) is staged as is:  As[row][64 depth bytes (+16 pad)]; an operand fragment
//   (16 depth bytes of one row per lane) is one ds_read_b128, conflict-free with the 80-byte row stride.
//   B (row-major, depth strided) is transposed on the way: a thread loads 16 depth rows x 4 columns (16 dwords,
//   each wave-wide load is contiguous along the columns), transposes 4x4 byte blocks in registers (v_perm_b32)
//   and stores, per column, the 16 consecutive depth bytes an MFMA lane needs:
//   Bs[depth block of 16][column%4][column/4][16 bytes] (+32 bytes pad per column%4 plane), so that both the
//   ds_write_b128 of the staging and the ds_read_b128 of the fragments are bank-conflict free.
// Both MFMA operands take 16 depth bytes per lane (lane%32 = row / column, lane/32 = which half of the 32 deep
// step); A and B use the same slot order, so the order of depth positions inside the instruction is immaterial.
// LDS is double buffered: the next depth step is fetched into registers while the current one is multiplied,
// written to the other buffer afterwards, one barrier per step.  Measured on 1024 x 50176 x 4608 the 256 x 128
// tile is the fastest of the three instances; the kernel is bound by the latency of the per-step global loads
// (one step of prefetch, one wave per SIMD), not by the matrix cores.
//
// Unsigned 8-bit operands with zero points (U8 = true; eq. (2) and (3) of the paper, the gemmlowp scheme): the
// bytes are re-biased to signed on the way in (x' = x - 128, one XOR), the matrix cores form sum a'b', and the
// epilogue applies  C = sum a'b' - zB' * rowsum(a') - zA' * colsum(b') + K * zA' * zB'  with zA' = zA - 128,
// zB' = zB - 128, which equals sum (a - zA)(b - zB).  Row and column sums are accumulated with packed dot products
// by the threads that stage the tiles, and combined through LDS after the depth loop.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BK = 64;
constexpr int A_STRIDE = BK + 16;  // bytes per staged A row

// rows = depth j, bytes = column i  ->  out[i] byte j = in[j] byte i
__device__ __forceinline__ void transpose4x4(const uint32_t r[4], uint32_t o[4])
{
    const uint32_t t0 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u);  // r0.b0 r1.b0 r0.b1 r1.b1
    const uint32_t t1 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);  // r0.b2 r1.b2 r0.b3 r1.b3
    const uint32_t t2 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
    o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

__device__ __forceinline__ int32_t bytesum(uint32_t x, int32_t c)
{
    return __builtin_amdgcn_sdot4((int)x, 0x01010101, c, false);
}

template <int TM, int TN, int MODE, bool U8>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2))) void gemm_i8_mfma_kernel(
    int M, int N, int K, const int8_t *__restrict__ A, int64_t lda, const int8_t *__restrict__ B, int64_t ldb,
    int32_t *__restrict__ C, int64_t ldc, int nMB, int nNB, int tiles_per_xcd, int zA, int zB)
{
    constexpr uint32_t FLIP = U8 ? 0x80808080u : 0u;  // unsigned byte -> signed byte minus 128
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int NQ = BN / 4;                       // column quads per tile
    constexpr int B_PLANE = NQ * 16 + 32;            // bytes per (depth block, column%4) plane
    constexpr int B_BLOCK = 4 * B_PLANE;             // bytes per depth block of 16
    constexpr int A_BYTES = BM * A_STRIDE, B_BYTES = 4 * B_BLOCK;
    constexpr int A_PT = BM * 4 / 256;               // uint4 loads of A per thread
    constexpr int B_UNITS = 4 * NQ;                  // (depth block, column quad) units
    constexpr int B_PT = (B_UNITS + 255) / 256;

    __shared__ __attribute__((aligned(16))) uint8_t smem[2][A_BYTES + B_BYTES];

    const int bid = blockIdx.x;
    const int idx = (bid & 7) * tiles_per_xcd + (bid >> 3);
    if ((bid >> 3) >= tiles_per_xcd || idx >= nMB * nNB)
        return;
    const int nb = idx / nMB, mb = idx - nb * nMB;  // the M blocks of one N block are adjacent: they share the B tile
    const int m0 = mb * BM, n0 = nb * BN;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave & 1, wn = wave >> 1;

    // one depth step of operands in flight from global memory
    uint4 a_pre[A_PT];
    uint32_t b_pre[B_PT][16];

    // Three ways to fetch a depth step, fixed per launch (MODE) so that the loads are straight-line code and the
    // compiler can count exactly how many may stay in flight (a load inside a branch makes it wait at once):
    //   0 raw      M, N, K multiples of the tile and aligned operands: no checks
    //   1 clamped  aligned operands with N % 4 == 0 and K % 16 == 0: addresses are clamped into range and
    //              out-of-range pieces replaced by zero
    //   2 bytes    anything else: guarded byte loads (slow, rare)
    auto fetch_raw = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const uint32_t *src = reinterpret_cast<const uint32_t *>(A + (int64_t)(m0 + (u >> 2)) * lda + k0 + (u & 3) * 16);
            // four dwords assembled by value (the compiler merges them into one 128-bit load); copying the uint4
            // as an aggregate makes the optimiser keep a_pre in memory and demote it to LDS
            a_pre[p] = make_uint4(src[0] ^ FLIP, src[1] ^ FLIP, src[2] ^ FLIP, src[3] ^ FLIP);
        }
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = (B_UNITS % 256 == 0) ? tid + p * 256 : (tid + p * 256) % B_UNITS;
            const int kb = u / NQ, nq = u % NQ;
            const int8_t *src = B + (int64_t)(k0 + kb * 16) * ldb + n0 + nq * 4;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                b_pre[p][j] = *reinterpret_cast<const uint32_t *>(src + (int64_t)j * ldb) ^ FLIP;
        }
    };
    auto fetch_clamped = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const int r = m0 + (u >> 2), k = k0 + (u & 3) * 16;
            const bool ok = r < M && k + 16 <= K;
            const int rr = r < M ? r : M - 1, kk = k + 16 <= K ? k : K - 16;
            const uint4 v = *reinterpret_cast<const uint4 *>(A + (int64_t)rr * lda + kk);
            a_pre[p] = ok ? make_uint4(v.x ^ FLIP, v.y ^ FLIP, v.z ^ FLIP, v.w ^ FLIP) : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = (B_UNITS % 256 == 0) ? tid + p * 256 : (tid + p * 256) % B_UNITS;
            const int kb = u / NQ, nq = u % NQ;
            const int n = n0 + nq * 4;
            const int nn = n + 4 <= N ? n : N - 4;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int k = k0 + kb * 16 + j;
                const int kk = k < K ? k : K - 1;
                const uint32_t x = *reinterpret_cast<const uint32_t *>(B + (int64_t)kk * ldb + nn);
                b_pre[p][j] = (k < K && n + 4 <= N) ? (x ^ FLIP) : 0u;
            }
        }
    };
    auto fetch_bytes = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const int r = m0 + (u >> 2), k = k0 + (u & 3) * 16;
            uint32_t w[4] = {0u, 0u, 0u, 0u};
            if (r < M)
                for (int i = 0; i < 16 && k + i < K; ++i)
                    w[i >> 2] |= (uint32_t)((uint8_t)A[(int64_t)r * lda + k + i] ^ (FLIP & 0xffu)) << (8 * (i & 3));
            a_pre[p] = make_uint4(w[0], w[1], w[2], w[3]);
        }
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = (B_UNITS % 256 == 0) ? tid + p * 256 : (tid + p * 256) % B_UNITS;
            const int kb = u / NQ, nq = u % NQ;
            const int n = n0 + nq * 4;
            for (int j = 0; j < 16; ++j) {
                const int k = k0 + kb * 16 + j;
                uint32_t x = 0u;
                if (k < K)
                    for (int i = 0; i < 4 && n + i < N; ++i)
                        x |= (uint32_t)((uint8_t)B[(int64_t)k * ldb + n + i] ^ (FLIP & 0xffu)) << (8 * i);
                b_pre[p][j] = x;
            }
        }
    };
    auto fetch = [&](int k0) __attribute__((always_inline)) {
        if constexpr (MODE == 0)
            fetch_raw(k0);
        else if constexpr (MODE == 1)
            fetch_clamped(k0);
        else
            fetch_bytes(k0);
    };
    // U8: signed sums of the staged bytes, per thread; the rows / columns a thread stages are the same in every step
    int32_t rs_acc[A_PT], cs_acc[B_PT][4];
#pragma unroll
    for (int p = 0; p < A_PT; ++p)
        rs_acc[p] = 0;
#pragma unroll
    for (int p = 0; p < B_PT; ++p)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            cs_acc[p][i] = 0;

    auto commit = [&](int buf) __attribute__((always_inline)) {
        uint8_t *As = smem[buf], *Bs = smem[buf] + A_BYTES;
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            *reinterpret_cast<uint4 *>(&As[(u >> 2) * A_STRIDE + (u & 3) * 16]) = a_pre[p];
            if constexpr (U8)
                rs_acc[p] = bytesum(a_pre[p].x, bytesum(a_pre[p].y, bytesum(a_pre[p].z, bytesum(a_pre[p].w, rs_acc[p]))));
        }
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = tid + p * 256;
            if (B_UNITS % 256 != 0 && u >= B_UNITS)
                continue;  // surplus threads fetched a duplicate unit; they do not store
            const int kb = u / NQ, nq = u % NQ;
            uint32_t o[4][4];  // o[q][i]: depth quad q, column i
#pragma unroll
            for (int q = 0; q < 4; ++q)
                transpose4x4(&b_pre[p][q * 4], o[q]);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                *reinterpret_cast<uint4 *>(&Bs[kb * B_BLOCK + i * B_PLANE + nq * 16]) =
                    make_uint4(o[0][i], o[1][i], o[2][i], o[3][i]);
                if constexpr (U8)
                    cs_acc[p][i] = bytesum(o[0][i], bytesum(o[1][i], bytesum(o[2][i], bytesum(o[3][i], cs_acc[p][i]))));
            }
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    auto compute = [&](int buf) __attribute__((always_inline)) {
        const uint8_t *As = smem[buf], *Bs = smem[buf] + A_BYTES;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i af[TM], bf[TN];
            const int kb = ks * 2 + (lane >> 5);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = (wm * TM + i) * 32 + (lane & 31);
                af[i] = *reinterpret_cast<const v4i *>(&As[row * A_STRIDE + kb * 16]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = (wn * TN + j) * 32 + (lane & 31);
                bf[j] = *reinterpret_cast<const v4i *>(&Bs[kb * B_BLOCK + (col & 3) * B_PLANE + (col >> 2) * 16]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    };

    // Software pipeline over depth steps: while step s is multiplied out of LDS buffer s%2 the loads of step s+1
    // are in flight; they are written to the other buffer afterwards.  One barrier per step.
    const int nsteps = (K + BK - 1) / BK;
    fetch(0);
    commit(0);
    __syncthreads();
    for (int s = 0; s < nsteps; ++s) {
        if (s + 1 < nsteps)
            fetch((s + 1) * BK);
        compute(s & 1);
        if (s + 1 < nsteps)
            commit((s + 1) & 1);
        __syncthreads();
    }

    // U8: combine the per-thread sums through LDS (the tile buffers are free after the last barrier):
    // rsum[row][4 depth quarters], csum[column][4 depth blocks]
    int32_t *rsum = reinterpret_cast<int32_t *>(&smem[0][0]);
    int32_t *csum = rsum + BM * 4;
    if constexpr (U8) {
        static_assert((BM + BN) * 4 * 4 <= 2 * (A_BYTES + B_BYTES), "sums must fit the tile buffers");
#pragma unroll
        for (int p = 0; p < A_PT; ++p)
            rsum[tid + p * 256] = rs_acc[p];                      // unit u = row*4 + quarter
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = tid + p * 256;
            if (B_UNITS % 256 != 0 && u >= B_UNITS)
                continue;
            const int kb = u / NQ, nq = u % NQ;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                csum[(nq * 4 + i) * 4 + kb] = cs_acc[p][i];
        }
        __syncthreads();
    }

    // accumulator layout of a 32x32 tile: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int lcol = (wn * TN + j) * 32 + (lane & 31);
            const int col = n0 + lcol;
            int32_t ccorr = 0;
            if constexpr (U8)
                ccorr = K * zA * zB - zA * (csum[lcol * 4] + csum[lcol * 4 + 1] + csum[lcol * 4 + 2] + csum[lcol * 4 + 3]);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lrow = (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int row = m0 + lrow;
                int32_t out = acc[i][j][r];
                if constexpr (U8)
                    out += ccorr - zB * (rsum[lrow * 4] + rsum[lrow * 4 + 1] + rsum[lrow * 4 + 2] + rsum[lrow * 4 + 3]);
                if (row < M && col < N)
                    C[(int64_t)row * ldc + col] = out;
            }
        }
}

template <int TM, int TN, bool U8>
hipError_t launch_tile(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                       int32_t *C, int64_t ldc, hipStream_t stream, int zA, int zB)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    const int nMB = (int)((M + BM - 1) / BM), nNB = (int)((N + BN - 1) / BN);
    const int64_t tiles = (int64_t)nMB * nNB;
    const int tiles_per_xcd = (int)((tiles + 7) / 8);
    const int64_t grid = (int64_t)tiles_per_xcd * 8;
    if (grid > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    const bool aligned = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(B) % 4 == 0) && (ldb % 4 == 0);
    const bool whole = (M % BM) == 0 && (N % BN) == 0 && (K % BK) == 0;
    const bool can_clamp = (N % 4) == 0 && (K % 16) == 0 && N >= 4 && K >= 16;
    const dim3 g((unsigned)grid), b(256);
    if (aligned && whole)
        hipLaunchKernelGGL((gemm_i8_mfma_kernel<TM, TN, 0, U8>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B,
                           ldb, C, ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    else if (aligned && can_clamp)
        hipLaunchKernelGGL((gemm_i8_mfma_kernel<TM, TN, 1, U8>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B,
                           ldb, C, ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    else
        hipLaunchKernelGGL((gemm_i8_mfma_kernel<TM, TN, 2, U8>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B,
                           ldb, C, ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    return hipGetLastError();
}

int g_i8_forced = -1;

}  // namespace

void i8_force_tile(int t) { g_i8_forced = t; }

hipError_t launch_gemm_i8(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                          int32_t *C, int64_t ldc, hipStream_t stream)
{
    // the 256 x 128 tile needs enough tiles to fill the 256 compute units; smaller problems use 128 x 128
    const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
    int t = g_i8_forced;
    // a right operand of at most 16 columns would leave a matrix-core tile almost empty: stream A with dot products
    if (t < 0 && N <= 16 && M >= 64)
        return launch_gemm_i8_skinny(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (t < 0)
        t = big_tiles >= 512 ? 2 : 0;
    if (t == 1)
        return launch_tile<4, 4, false>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
    if (t == 2)
        return launch_tile<4, 2, false>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
    return launch_tile<2, 2, false>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
}

// unsigned operands with zero points; zA, zB in [0, 255]
hipError_t launch_gemm_u8(int64_t M, int64_t N, int64_t K, const uint8_t *A, int64_t lda, const uint8_t *B, int64_t ldb,
                          int zA, int zB, int32_t *C, int64_t ldc, hipStream_t stream)
{
    const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
    const int8_t *a = reinterpret_cast<const int8_t *>(A), *b = reinterpret_cast<const int8_t *>(B);
    if (big_tiles >= 512)
        return launch_tile<4, 2, true>(M, N, K, a, lda, b, ldb, C, ldc, stream, zA - 128, zB - 128);
    return launch_tile<2, 2, true>(M, N, K, a, lda, b, ldb, C, ldc, stream, zA - 128, zB - 128);
}

}  // namespace lowbit
