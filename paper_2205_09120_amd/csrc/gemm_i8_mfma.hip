// int8 x int8 -> int32 GEMM on the gfx950 integer matrix cores (v_mfma_i32_32x32x32_i8).
//
// Comparison point for the popcount kernels: it computes the same C = A B from unpacked int8 operands, the role
// the 8-bit gemmlowp multiplication (U8) plays in Section IV of the paper.
//
// Three kernels.  The first two share the tile layouts described here.  gemm_i8_mfma_kernel: workgroup = 4 waves in
// a 2 x 2 arrangement; a wave computes TM x TN MFMA tiles of 32 x 32, so the workgroup tile is (64*TM) x (64*TN);
// depth step 64 (two MFMA depth steps of 32); instances 128 x 128 (TM=TN=2, what unaligned operands fall back to),
// 256 x 128 and 256 x 256 (selectable).  gemm_i8_ws_kernel (further down): the 256 x 128 tile with the loading and
// the multiplying done by different waves.  gemm_i8_dl_kernel (last): operands go from global memory straight into
// LDS; the default for aligned operands of any size.
//   A (row-major, depth contiguous) is staged as is:  As[row][64 depth bytes (+16 pad)]; an operand fragment
//   (16 depth bytes of one row per lane) is one ds_read_b128, conflict-free with the 80-byte row stride.
//   B (row-major, depth strided) is transposed on the way: a thread loads 16 depth rows x 4 columns (16 dwords,
//   each wave-wide load is contiguous along the columns), transposes 4x4 byte blocks in registers (v_perm_b32)
//   and stores, per column, the 16 consecutive depth bytes an MFMA lane needs:
//   Bs[depth block of 16][column%4][column/4][16 bytes] (+64 bytes pad per column%4 plane, so that the four
//   planes start 16 banks apart): the ds_write_b128 of the staging and the ds_read_b128 of the fragments both
//   spread over all banks.
// Both MFMA operands take 16 depth bytes per lane (lane%32 = row / column, lane/32 = which half of the 32 deep
// step); A and B use the same slot order, so the order of depth positions inside the instruction is immaterial.
// LDS is double buffered: in the 4-wave kernel the next depth step is fetched into registers while the current one
// is multiplied and written to the other buffer afterwards, one barrier per step.
//
// Unsigned 8-bit operands with zero points (U8 = true; eq. (2) and (3) of the paper, the gemmlowp scheme): the
// bytes are re-biased to signed on their way into LDS (x' = x - 128, one XOR), the matrix cores form sum a'b', and
// the epilogue applies  C = sum a'b' - zB' * rowsum(a') - zA' * colsum(b') + K * zA' * zB'  with zA' = zA - 128,
// zB' = zB - 128, which equals sum (a - zA)(b - zB).  Row and column sums are taken by the threads that stage the
// tiles, as sums of the unsigned bytes (v_sad_u8 against zero, 4 bytes per instruction) minus 128 per byte, and
// combined through LDS after the depth loop.
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>

#include <type_traits>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
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

// c + sum of the four unsigned bytes of x, one full-rate instruction (the packed dot product that would add signed
// bytes directly issues at a fraction of that rate and slowed the whole kernel down by a factor of two)
__device__ __forceinline__ uint32_t bytesum(uint32_t x, uint32_t c) { return __builtin_amdgcn_sad_u8(x, 0u, c); }

// LDS bytes of one of the two staging buffers of a 64*TM x 64*TN tile
template <int TM, int TN> struct I8TileLds {
    static constexpr int A_BYTES = 64 * TM * A_STRIDE;
    static constexpr int B_BYTES = 4 * 4 * ((64 * TN / 4) * 16 + 64);
    static constexpr int STAGE = A_BYTES + B_BYTES;
};

// One workgroup tile (block row mb, block column nb) of C = A B; smem_base: two staging buffers of I8TileLds::STAGE bytes.
template <int TM, int TN, int MODE, bool U8>
__device__ __forceinline__ void gemm_i8_tile(int M, int N, int K, const int8_t *__restrict__ A, int64_t lda,
                                             const int8_t *__restrict__ B, int64_t ldb, int32_t *__restrict__ C,
                                             int64_t ldc, int mb, int nb, int zA, int zB, uint8_t *smem_base)
{
    constexpr uint32_t FLIP = U8 ? 0x80808080u : 0u;  // unsigned byte -> signed byte minus 128
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int NQ = BN / 4;                       // column quads per tile
    constexpr int B_PLANE = NQ * 16 + 64;            // bytes per (depth block, column%4) plane
    constexpr int B_BLOCK = 4 * B_PLANE;             // bytes per depth block of 16
    constexpr int A_BYTES = BM * A_STRIDE, B_BYTES = 4 * B_BLOCK;
    constexpr int A_PT = BM * 4 / 256;               // uint4 loads of A per thread
    constexpr int B_UNITS = 4 * NQ;                  // (depth block, column quad) units
    constexpr int B_PT = (B_UNITS + 255) / 256;
    static_assert(A_BYTES == I8TileLds<TM, TN>::A_BYTES && B_BYTES == I8TileLds<TM, TN>::B_BYTES, "LDS layout");

    uint8_t(*smem)[A_BYTES + B_BYTES] = reinterpret_cast<uint8_t(*)[A_BYTES + B_BYTES]>(smem_base);
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
    //   2 overlap  any alignment and any M, N >= 4, K >= 64: the last depth step starts at K - 64 and the depth
    //              positions it shares with the step before are zeroed in A; a column quad that sticks out over N is
    //              fetched from N - 4 and stored to the columns it really holds; loads go through memcpy, which the
    //              compiler turns into dword / dwordx4 loads that need no alignment
    //   3 bytes    N < 4 or K < 64: guarded byte loads (slow, tiny problems only)
    auto fetch_raw = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const uint32_t *src = reinterpret_cast<const uint32_t *>(A + (int64_t)(m0 + (u >> 2)) * lda + k0 + (u & 3) * 16);
            // four dwords assembled by value (the compiler merges them into one 128-bit load); copying the uint4
            // as an aggregate makes the optimiser keep a_pre in memory and demote it to LDS
            a_pre[p] = make_uint4(src[0], src[1], src[2], src[3]);
        }
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = (B_UNITS % 256 == 0) ? tid + p * 256 : (tid + p * 256) % B_UNITS;
            const int kb = u / NQ, nq = u % NQ;
            const int8_t *src = B + (int64_t)(k0 + kb * 16) * ldb + n0 + nq * 4;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                b_pre[p][j] = *reinterpret_cast<const uint32_t *>(src + (int64_t)j * ldb);
        }
    };
    // clamped: the loads only (addresses forced into range); what lies out of range is replaced by zero when the
    // step is committed, so that no load is followed by a use that would make the wave wait for it at once
    auto fetch_clamped = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const int r = m0 + (u >> 2), k = k0 + (u & 3) * 16;
            const int rr = r < M ? r : M - 1, kk = k + 16 <= K ? k : K - 16;
            const uint32_t *src = reinterpret_cast<const uint32_t *>(A + (int64_t)rr * lda + kk);
            a_pre[p] = make_uint4(src[0], src[1], src[2], src[3]);
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
                b_pre[p][j] = *reinterpret_cast<const uint32_t *>(B + (int64_t)kk * ldb + nn);
            }
        }
    };
    auto mask_clamped = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const int r = m0 + (u >> 2), k = k0 + (u & 3) * 16;
            if (!(r < M && k + 16 <= K))
                a_pre[p] = make_uint4(FLIP, FLIP, FLIP, FLIP);
        }
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = (B_UNITS % 256 == 0) ? tid + p * 256 : (tid + p * 256) % B_UNITS;
            const int kb = u / NQ, nq = u % NQ;
            const bool n_ok = n0 + nq * 4 + 4 <= N;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                b_pre[p][j] = (n_ok && k0 + kb * 16 + j < K) ? b_pre[p][j] : FLIP;
        }
    };
    const int nsteps = (K + BK - 1) / BK;
    // first depth position of step s (mode 2: the last step is shifted back so that it ends at K)
    auto kstart = [&](int s) { return (MODE == 2 && s == nsteps - 1) ? K - BK : s * BK; };
    auto fetch_overlap = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const int r = m0 + (u >> 2);
            const int rr = r < M ? r : M - 1;
            __builtin_memcpy(&a_pre[p], A + (int64_t)rr * lda + k0 + (u & 3) * 16, 16);
        }
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = (B_UNITS % 256 == 0) ? tid + p * 256 : (tid + p * 256) % B_UNITS;
            const int kb = u / NQ, nq = u % NQ;
            const int n = n0 + nq * 4;
            const int nn = n + 4 <= N ? n : N - 4;
            const int8_t *src = B + (int64_t)(k0 + kb * 16) * ldb + nn;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                __builtin_memcpy(&b_pre[p][j], src + (int64_t)j * ldb, 4);
        }
    };
    // last step of mode 2: its first `cut` depth positions were already multiplied by the step before
    auto mask_overlap = [&](int s) __attribute__((always_inline)) {
        const int cut = s == nsteps - 1 ? (nsteps - 1) * BK - (K - BK) : 0;
        if (cut <= 0)
            return;
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const int z = cut - (u & 3) * 16;  // leading bytes of this 16-byte piece to zero
            uint32_t w[4] = {a_pre[p].x, a_pre[p].y, a_pre[p].z, a_pre[p].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int nz = z - 4 * j;
                const uint32_t m = nz >= 4 ? 0xffffffffu : nz <= 0 ? 0u : ((1u << (8 * nz)) - 1u);
                w[j] = (w[j] & ~m) | (FLIP & m);
            }
            a_pre[p] = make_uint4(w[0], w[1], w[2], w[3]);
        }
        if constexpr (U8) {  // the column sums must not count those rows twice either
#pragma unroll
            for (int p = 0; p < B_PT; ++p) {
                const int u = (B_UNITS % 256 == 0) ? tid + p * 256 : (tid + p * 256) % B_UNITS;
                const int kb = u / NQ;
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    b_pre[p][j] = kb * 16 + j < cut ? FLIP : b_pre[p][j];
            }
        }
    };
    auto fetch_bytes = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const int r = m0 + (u >> 2), k = k0 + (u & 3) * 16;
            uint32_t w[4] = {FLIP, FLIP, FLIP, FLIP};
            if (r < M)
                for (int i = 0; i < 16 && k + i < K; ++i)
                    w[i >> 2] ^= (uint32_t)((uint8_t)A[(int64_t)r * lda + k + i] ^ (FLIP & 0xffu)) << (8 * (i & 3));
            a_pre[p] = make_uint4(w[0], w[1], w[2], w[3]);
        }
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = (B_UNITS % 256 == 0) ? tid + p * 256 : (tid + p * 256) % B_UNITS;
            const int kb = u / NQ, nq = u % NQ;
            const int n = n0 + nq * 4;
            for (int j = 0; j < 16; ++j) {
                const int k = k0 + kb * 16 + j;
                uint32_t x = FLIP;
                if (k < K)
                    for (int i = 0; i < 4 && n + i < N; ++i)
                        x ^= (uint32_t)((uint8_t)B[(int64_t)k * ldb + n + i] ^ (FLIP & 0xffu)) << (8 * i);
                b_pre[p][j] = x;
            }
        }
    };
    auto fetch = [&](int k0) __attribute__((always_inline)) {
        if constexpr (MODE == 0)
            fetch_raw(k0);
        else if constexpr (MODE == 1)
            fetch_clamped(k0);
        else if constexpr (MODE == 2)
            fetch_overlap(k0);
        else
            fetch_bytes(k0);
    };
    // U8: sums of the staged bytes as UNSIGNED values, per thread; the rows / columns a thread stages are the same in
    // every step and every step adds exactly 16 bytes per sum (out-of-range bytes count as 128), so the sum of the
    // re-biased signed bytes is the unsigned sum minus 128 * 16 * steps.
    uint32_t rs_acc[A_PT], cs_acc[B_PT][4];
#pragma unroll
    for (int p = 0; p < A_PT; ++p)
        rs_acc[p] = 0;
#pragma unroll
    for (int p = 0; p < B_PT; ++p)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            cs_acc[p][i] = 0;

    auto commit = [&](int s) __attribute__((always_inline)) {
        const int buf = s & 1;
        uint8_t *As = smem[buf], *Bs = smem[buf] + A_BYTES;
        if constexpr (MODE == 1)
            mask_clamped(s * BK);
        if constexpr (MODE == 2)
            mask_overlap(s);
#pragma unroll
        for (int p = 0; p < A_PT; ++p) {
            const int u = tid + p * 256;
            const uint4 v = a_pre[p];
            *reinterpret_cast<uint4 *>(&As[(u >> 2) * A_STRIDE + (u & 3) * 16]) =
                make_uint4(v.x ^ FLIP, v.y ^ FLIP, v.z ^ FLIP, v.w ^ FLIP);
            if constexpr (U8)
                rs_acc[p] = bytesum(v.x, bytesum(v.y, bytesum(v.z, bytesum(v.w, rs_acc[p]))));
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
                    make_uint4(o[0][i] ^ FLIP, o[1][i] ^ FLIP, o[2][i] ^ FLIP, o[3][i] ^ FLIP);
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
    fetch(kstart(0));
    commit(0);
    __syncthreads();
    for (int s = 0; s < nsteps; ++s) {
        if (s + 1 < nsteps)
            fetch(kstart(s + 1));
        compute(s & 1);
        if (s + 1 < nsteps)
            commit(s + 1);
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
            rsum[tid + p * 256] = (int32_t)rs_acc[p] - 2048 * nsteps;  // unit u = row*4 + quarter
#pragma unroll
        for (int p = 0; p < B_PT; ++p) {
            const int u = tid + p * 256;
            if (B_UNITS % 256 != 0 && u >= B_UNITS)
                continue;
            const int kb = u / NQ, nq = u % NQ;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                csum[(nq * 4 + i) * 4 + kb] = (int32_t)cs_acc[p][i] - 2048 * nsteps;
        }
        __syncthreads();
    }

    // accumulator layout of a 32x32 tile: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int lcol = (wn * TN + j) * 32 + (lane & 31);
            int col = n0 + lcol;
            bool col_ok = col < N;
            if constexpr (MODE == 2) {
                // a quad that sticks out over N was fetched from column N - 4: its slots hold columns N-4 .. N-1;
                // those below the quad's own first column belong to the quad before and are not stored again
                const int nq0 = n0 + (lcol & ~3);
                if (nq0 + 4 > N) {
                    col = N - 4 + (lcol & 3);
                    col_ok = nq0 < N && col >= nq0;
                }
            }
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
                if (row < M && col_ok)
                    C[(int64_t)row * ldc + col] = out;
            }
        }
}

template <int TM, int TN, int MODE, bool U8>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2))) void gemm_i8_mfma_kernel(
    int M, int N, int K, const int8_t *__restrict__ A, int64_t lda, const int8_t *__restrict__ B, int64_t ldb,
    int32_t *__restrict__ C, int64_t ldc, int nMB, int nNB, int tiles_per_xcd, int zA, int zB)
{
    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * I8TileLds<TM, TN>::STAGE];
    const int bid = blockIdx.x;
    const int idx = (bid & 7) * tiles_per_xcd + (bid >> 3);
    if ((bid >> 3) >= tiles_per_xcd || idx >= nMB * nNB)
        return;
    const int nb = idx / nMB, mb = idx - nb * nMB;  // the M blocks of one N block are adjacent: they share the B tile
    gemm_i8_tile<TM, TN, MODE, U8>(M, N, K, A, lda, B, ldb, C, ldc, mb, nb, zA, zB, smem);
}

// Grouped launch of the comparator: `count` independent products in one grid of 64 x 64 tiles.  The table (built on
// the host) maps each workgroup id to a problem record; the record carries the fetch mode the single-product launcher
// would pick for that problem.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2))) void gemm_i8_group_kernel(
    const I8GroupHeader *__restrict__ table, uint32_t count)
{
    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * I8TileLds<1, 1>::STAGE];
    const uint32_t bid = blockIdx.x;
    if (table->magic != kI8GroupMagic || table->count != count || table->workgroups != gridDim.x)
        return;
    const I8GroupRecord *__restrict__ recs = reinterpret_cast<const I8GroupRecord *>(table + 1);
    const uint32_t *__restrict__ owner = reinterpret_cast<const uint32_t *>(recs + count);
    const uint32_t p = owner[bid];
    if (p >= count)
        return;
    const I8GroupRecord r = recs[p];
    const int local = (int)(bid - r.tile0);
    const int nb = local / r.nMB, mb = local - nb * r.nMB;
    switch (r.mode) {
    case 0: gemm_i8_tile<1, 1, 0, false>(r.M, r.N, r.K, r.A, r.lda, r.B, r.ldb, r.C, r.ldc, mb, nb, 0, 0, smem); break;
    case 1: gemm_i8_tile<1, 1, 1, false>(r.M, r.N, r.K, r.A, r.lda, r.B, r.ldb, r.C, r.ldc, mb, nb, 0, 0, smem); break;
    case 2: gemm_i8_tile<1, 1, 2, false>(r.M, r.N, r.K, r.A, r.lda, r.B, r.ldb, r.C, r.ldc, mb, nb, 0, 0, smem); break;
    default: gemm_i8_tile<1, 1, 3, false>(r.M, r.N, r.K, r.A, r.lda, r.B, r.ldb, r.C, r.ldc, mb, nb, 0, 0, smem); break;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Wave-specialised instance for large problems: 256 x 128 tile, 8 waves.
//
// The kernel above keeps one depth step of operands in flight per wave, and a wave that multiplies cannot afford the
// registers for more (128 accumulator registers per lane); with a global-load latency several times the 0.2 us a
// depth step takes on the matrix cores, the matrix cores wait.  Here the two jobs are split between waves of one
// workgroup, two waves per SIMD:
//   waves 0-3 (consumers)  only read operand fragments from LDS and issue MFMAs (2 x 2 arrangement, 128 x 64 outputs
//                          each), fragment reads of the next half step overlapping the MFMAs of the current one;
//   waves 4-5 (B loaders)  fetch B (depth-strided), transpose 4x4 byte blocks in registers and write the LDS layout
//                          the fragments need;  waves 6-7 (A loaders) fetch and store A.
// Loaders own no accumulators, so they keep DEPTH depth steps of loads in flight in registers.  LDS is double
// buffered; barrier k (k = 0 .. steps-1) means "buffer k%2 holds depth step k".  A consumer finishes its reads of
// step k before it arrives at barrier k+1, and a loader overwrites buffer k%2 (with step k+2) only after it has
// passed barrier k+1, so two buffers suffice.  Barriers are a bare s_barrier after waiting for the wave's own LDS
// operations only: a full __syncthreads() would also wait for the loaders' outstanding global loads and undo the
// prefetch.  Unsigned operands: the loaders also form the row / column sums of eq. (3) (they have the registers to
// spare), so the consumers' loop is the same as for signed operands.
__device__ __forceinline__ void lds_barrier()
{
    // the scheduling fences keep register-only work (the byte transposes of a later step, MFMAs) on its side of the
    // barrier: moved above it, a transpose would wait for loads that are meant to stay in flight
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0) only; as a builtin, so that the compiler's own counting sees it
    asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

template <int MODE, bool U8, int DEPTH>
__global__ __launch_bounds__(512) void gemm_i8_ws_kernel(int M, int N, int K, const int8_t *__restrict__ A, int64_t lda,
                                                         const int8_t *__restrict__ B, int64_t ldb,
                                                         int32_t *__restrict__ C, int64_t ldc, int nMB, int nNB,
                                                         int tiles_per_xcd, int zA, int zB)
{
    static_assert(MODE == 0 || MODE == 1, "raw or clamped fetch only");
    constexpr uint32_t FLIP = U8 ? 0x80808080u : 0u;
    constexpr int TM = 4, TN = 2;
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int NQ = BN / 4;
    constexpr int B_PLANE = NQ * 16 + 64;
    constexpr int B_BLOCK = 4 * B_PLANE;
    constexpr int A_BYTES = BM * A_STRIDE, B_BYTES = 4 * B_BLOCK;
    constexpr int A_PT = BM * 4 / 128;  // uint4 loads of A per A-loader thread (128 of them)
    static_assert(4 * NQ == 128, "one B unit per B-loader thread");

    __shared__ __attribute__((aligned(16))) uint8_t smem[2][A_BYTES + B_BYTES];
    __shared__ int32_t sums[U8 ? (BM + BN) * 4 : 1];  // rsum[row][4 depth quarters], csum[column][4 depth blocks]

    const int bid = blockIdx.x;
    const int idx = (bid & 7) * tiles_per_xcd + (bid >> 3);
    if ((bid >> 3) >= tiles_per_xcd || idx >= nMB * nNB)
        return;
    const int nb = idx / nMB, mb = idx - nb * nMB;
    const int m0 = mb * BM, n0 = nb * BN;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nsteps = (K + BK - 1) / BK;
    int32_t *rsum = sums, *csum = sums + (U8 ? BM * 4 : 0);

    if (wave >= 6) {
        // ------------------------------------------------------------------ A loaders
        const int t = tid - 384;  // 0..127
        uint4 pre[DEPTH][A_PT];
        uint32_t rs_acc[A_PT];  // unsigned byte sums, 16 bytes per step each (see the 4-wave kernel)
#pragma unroll
        for (int p = 0; p < A_PT; ++p)
            rs_acc[p] = 0;
        // loads of a step beyond the last one re-read the last step (never used): no load sits under a branch
        auto load = [&](uint4(&dst)[A_PT], int step) __attribute__((always_inline)) {
            const int k0 = (step < nsteps ? step : nsteps - 1) * BK;
#pragma unroll
            for (int p = 0; p < A_PT; ++p) {
                const int u = t + p * 128;
                const int r = m0 + (u >> 2), k = k0 + (u & 3) * 16;
                if constexpr (MODE == 0) {
                    const uint32_t *src = reinterpret_cast<const uint32_t *>(A + (int64_t)r * lda + k);
                    dst[p] = make_uint4(src[0], src[1], src[2], src[3]);
                } else {
                    // out-of-range pieces are replaced by zero at commit time, not here: a use right behind the
                    // load would make the wave wait for it at once
                    const int rr = r < M ? r : M - 1, kk = k + 16 <= K ? k : K - 16;
                    const uint32_t *src = reinterpret_cast<const uint32_t *>(A + (int64_t)rr * lda + kk);
                    dst[p] = make_uint4(src[0], src[1], src[2], src[3]);
                }
            }
        };
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            load(pre[d], d);
        auto commit = [&](const uint4(&src)[A_PT], int step) __attribute__((always_inline)) {
            uint8_t *As = smem[step & 1];
#pragma unroll
            for (int p = 0; p < A_PT; ++p) {
                const int u = t + p * 128;
                uint4 v = src[p];
                if constexpr (MODE == 1) {
                    if (!(m0 + (u >> 2) < M && step * BK + (u & 3) * 16 + 16 <= K))
                        v = make_uint4(FLIP, FLIP, FLIP, FLIP);
                }
                *reinterpret_cast<uint4 *>(&As[(u >> 2) * A_STRIDE + (u & 3) * 16]) =
                    make_uint4(v.x ^ FLIP, v.y ^ FLIP, v.z ^ FLIP, v.w ^ FLIP);
                if constexpr (U8)
                    rs_acc[p] = bytesum(v.x, bytesum(v.y, bytesum(v.z, bytesum(v.w, rs_acc[p]))));
            }
        };
        // Groups of DEPTH steps with compile-time slot numbers and no branch inside, so that the compiler's count of
        // loads that may stay in flight at each use is exact; the last nsteps % DEPTH steps need no further loads.
        const int full = nsteps / DEPTH * DEPTH;
        int s0 = 0;
        for (; s0 < full; s0 += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                commit(pre[d], s0 + d);
                load(pre[d], s0 + d + DEPTH);
                lds_barrier();
            }
        }
#pragma unroll
        for (int d = 0; d + 1 < DEPTH; ++d)
            if (s0 + d < nsteps) {
                commit(pre[d], s0 + d);
                lds_barrier();
            }
        if constexpr (U8) {
#pragma unroll
            for (int p = 0; p < A_PT; ++p)
                rsum[t + p * 128] = (int32_t)rs_acc[p] - 2048 * nsteps;  // unit u = row*4 + quarter
            lds_barrier();
        }
        return;
    }
    if (wave >= 4) {
        // ------------------------------------------------------------------ B loaders
        const int u = tid - 256;  // 0..127: one (depth block of 16, column quad) unit
        const int kb = u / NQ, nq = u % NQ;
        uint32_t pre[DEPTH][16];
        uint32_t cs_acc[4] = {0u, 0u, 0u, 0u};
        auto load = [&](uint32_t(&dst)[16], int step) __attribute__((always_inline)) {
            const int k0 = (step < nsteps ? step : nsteps - 1) * BK + kb * 16;
            const int n = n0 + nq * 4;
            if constexpr (MODE == 0) {
                const int8_t *src = B + (int64_t)k0 * ldb + n;
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    dst[j] = *reinterpret_cast<const uint32_t *>(src + (int64_t)j * ldb);
            } else {
                const int nn = n + 4 <= N ? n : N - 4;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int k = k0 + j;
                    const int kk = k < K ? k : K - 1;
                    dst[j] = *reinterpret_cast<const uint32_t *>(B + (int64_t)kk * ldb + nn);  // masked at commit
                }
            }
        };
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            load(pre[d], d);
        auto commit = [&](const uint32_t(&src)[16], int step) __attribute__((always_inline)) {
            uint8_t *Bs = smem[step & 1] + A_BYTES;
            uint32_t o[4][4];  // o[q][i]: depth quad q, column i
            if constexpr (MODE == 1) {
                uint32_t m[16];
                const bool n_ok = n0 + nq * 4 + 4 <= N;
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    m[j] = (n_ok && step * BK + kb * 16 + j < K) ? src[j] : FLIP;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    transpose4x4(&m[q * 4], o[q]);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    transpose4x4(&src[q * 4], o[q]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                *reinterpret_cast<uint4 *>(&Bs[kb * B_BLOCK + i * B_PLANE + nq * 16]) =
                    make_uint4(o[0][i] ^ FLIP, o[1][i] ^ FLIP, o[2][i] ^ FLIP, o[3][i] ^ FLIP);
                if constexpr (U8)
                    cs_acc[i] = bytesum(o[0][i], bytesum(o[1][i], bytesum(o[2][i], bytesum(o[3][i], cs_acc[i]))));
            }
        };
        const int full = nsteps / DEPTH * DEPTH;
        int s0 = 0;
        for (; s0 < full; s0 += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                commit(pre[d], s0 + d);
                load(pre[d], s0 + d + DEPTH);
                lds_barrier();
            }
        }
#pragma unroll
        for (int d = 0; d + 1 < DEPTH; ++d)
            if (s0 + d < nsteps) {
                commit(pre[d], s0 + d);
                lds_barrier();
            }
        if constexpr (U8) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                csum[(nq * 4 + i) * 4 + kb] = (int32_t)cs_acc[i] - 2048 * nsteps;
            lds_barrier();
        }
        return;
    }

    // ---------------------------------------------------------------------- consumers
    const int wm = wave & 1, wn = wave >> 1;
    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    auto read_frags = [&](int buf, int ks, v4i(&af)[TM], v4i(&bf)[TN]) __attribute__((always_inline)) {
        const uint8_t *As = smem[buf], *Bs = smem[buf] + A_BYTES;
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
    };
    auto mfma_all = [&](const v4i(&af)[TM], const v4i(&bf)[TN]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
    };

    v4i fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    lds_barrier();  // barrier 0
    read_frags(0, 0, fa0, fb0);
    // The scheduling fences pin "issue the fragment reads of the next half step, then the 8 MFMAs of this one":
    // left alone, the scheduler sinks the reads below the MFMAs to reuse the fragment registers, and the LDS
    // latency is then exposed twice per step.
    for (int s = 0; s + 1 < nsteps; ++s) {
        read_frags(s & 1, 1, fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_all(fa0, fb0);
        lds_barrier();  // barrier s+1; every read of buffer s%2 has completed
        read_frags((s + 1) & 1, 0, fa0, fb0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_all(fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);
    }
    read_frags((nsteps - 1) & 1, 1, fa1, fb1);  // last step, peeled so that the loop body has no branch
    __builtin_amdgcn_sched_barrier(0);
    mfma_all(fa0, fb0);
    mfma_all(fa1, fb1);
    if constexpr (U8)
        lds_barrier();  // the sums are in LDS

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int lcol = (wn * TN + j) * 32 + (lane & 31);
            int col = n0 + lcol;
            bool col_ok = col < N;
            if constexpr (MODE == 2) {
                // a quad that sticks out over N was fetched from column N - 4: its slots hold columns N-4 .. N-1;
                // those below the quad's own first column belong to the quad before and are not stored again
                const int nq0 = n0 + (lcol & ~3);
                if (nq0 + 4 > N) {
                    col = N - 4 + (lcol & 3);
                    col_ok = nq0 < N && col >= nq0;
                }
            }
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
                if (MODE == 0 || (row < M && col < N))
                    C[(int64_t)row * ldc + col] = out;
            }
        }
}

// ---------------------------------------------------------------------------------------------------------------
// Direct-to-LDS kernel, the default whenever every 16-byte chunk of the operands is aligned: 8 waves, tile
// (64*TM) x (64*TN) with instances 256 x 128 (large problems), 128 x 128 and 64 x 64 (small ones, where more and
// smaller workgroups hide the latency of a short depth loop better).
//
// In the kernels above every operand byte crosses the register file twice (global -> VGPR -> LDS -> VGPR), and the
// returns of the global loads and of the LDS fragment reads share the way into the registers: measured on the
// wave-specialised kernel, global loads alone or fragment reads alone take half the time the two take together.
// Here global memory is read straight into LDS (global_load_lds_dwordx4: lane l of a wave-wide load writes 16 bytes
// at LDS base + 16*l), so only fragments enter registers:
//   A tile  [row][BKB depth bytes]; the 16-byte chunk c of a row is stored at slot c ^ f(row), f chosen so that the
//           ds_read_b128 of an MFMA A fragment (32 consecutive rows, one chunk) spreads over all banks.  With
//           BKB = 128 a row of the tile is one whole 128-byte cache line of A; half lines (BKB = 64) move through
//           the caches at about half the rate, which is why the 128-byte stage is the default.
//   B tile  [depth row][64*TN column bytes] as in memory (no transpose on the way in), chunk c of depth row r stored
//           at slot c ^ (r & 7) (128 columns) or c ^ ((r >> 2) & 3) (64 columns).  The MFMA B fragment (16 depth bytes of one column per lane) is read with the
//           transposing LDS read ds_read_b64_tr_b8: 16 lanes hand in the addresses of 8 rows x 16 bytes (lanes 2m and
//           2m+1 the two halves of row m) and lane i receives byte i of each of the 8 rows.
// The swizzles cost nothing: a lane of a direct load may fetch any global chunk, only its LDS slot is fixed.
// Waves 0-3 multiply as in the wave-specialised kernel; waves 4-7 issue the direct loads (no data registers),
// STAGES - 1 depth stages ahead through a ring of STAGES LDS stages.  Barrier k means "stage k % STAGES holds depth
// step k"; a loader waits for its own loads of step k (vmcnt) before barrier k and refills the stage of step k - 1
// after it, which every consumer has finished reading by then.  Unsigned operands (U8): the bytes cannot be re-biased
// on the way in, so the consumers do it on the fragments and also take the byte sums of eq. (3) from them.
// RAGGED: rows beyond M and column chunks beyond N are fetched from the last valid row / chunk instead (always in
// bounds; the products they feed are never stored) and the stores are guarded; N must be a multiple of 16.
template <int STAGES, int BKB, bool U8, int TM, int TN, bool RAGGED>
__global__ __launch_bounds__(512) void gemm_i8_dl_kernel(int M, int N, int K, const int8_t *__restrict__ A, int64_t lda,
                                                         const int8_t *__restrict__ B, int64_t ldb,
                                                         int32_t *__restrict__ C, int64_t ldc, int nMB, int nNB,
                                                         int tiles_per_xcd, int zA, int zB)
{
    constexpr uint32_t FLIP = U8 ? 0x80808080u : 0u;  // unsigned byte -> signed byte minus 128
    constexpr int BM = 64 * TM, BN = 64 * TN;             // 2 x 2 consumer waves of TM x TN MFMA tiles each
    constexpr int KS = BKB / 32;                          // MFMA depth steps per stage
    constexpr int CA = BKB / 16;                          // 16-byte chunks per A row
    constexpr int RA = 64 / CA;                           // A rows per wave-wide load
    constexpr int SH = CA == 4 ? 2 : 1;                   // A slot swizzle: chunk ^ ((row >> SH) & (CA - 1))
    constexpr int CB = BN / 16;                           // 16-byte chunks per B row
    constexpr int RB = 64 / CB;                           // B depth rows per wave-wide load
    constexpr int A_BYTES = BM * BKB, B_BYTES = BKB * BN;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int A_LOADS = A_BYTES / 1024 / 4, B_LOADS = B_BYTES / 1024 / 4;  // per loader wave and step
    constexpr int LOADS = A_LOADS + B_LOADS;
    static_assert((BKB == 64 || BKB == 128) && (CB == 4 || CB == 8) && A_LOADS >= 1 && B_LOADS >= 1,
                  "tile shapes the slot arithmetic below covers");
    // B slot swizzle: chunk c of depth row r sits in slot c ^ fB(r); eight consecutive rows must land on different
    // bank groups for the transposing read (row stride 128 bytes: r & 7; 64 bytes: (r >> 2) & 3)
    auto fB = [](int r) { return CB == 8 ? (r & 7) : ((r >> 2) & 3); };

    __shared__ __attribute__((aligned(1024))) uint8_t smem[STAGES * STAGE];
    __shared__ uint32_t sums[U8 ? (BM + BN) * 2 : 1];  // U8: unsigned byte sums, [row or column][depth half of the lane]

    const int bid = blockIdx.x;
    const int idx = (bid & 7) * tiles_per_xcd + (bid >> 3);
    if ((bid >> 3) >= tiles_per_xcd || idx >= nMB * nNB)
        return;
    const int nb = idx / nMB, mb = idx - nb * nMB;
    const int m0 = mb * BM, n0 = nb * BN;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nsteps = K / BKB;

    if (wave >= 4) {
        // ------------------------------------------------------------------ loaders
        const int w = wave - 4;
        // A: wave-wide load q covers rows RA*q .. RA*q+RA-1; this wave issues q = A_LOADS*w .. A_LOADS*w + A_LOADS-1.
        // With 8 chunks per row the swizzle term (row >> 1) & 7 has a bit that alternates with q.
        // B: wave-wide load q covers depth rows RB*q .. RB*q+RB-1; this wave issues q = B_LOADS*w .. + B_LOADS-1.
        // Ragged tiles: rows / column chunks beyond the matrix re-read the last valid ones (their products are
        // never stored); the depth is always whole.
        const int a_row = lane / CA, a_slot = lane % CA;
        const int b_row = lane / CB, b_slot = lane % CB;
        const int8_t *pa0[A_LOADS], *pb0[B_LOADS];
#pragma unroll
        for (int q = 0; q < A_LOADS; ++q) {
            const int rl = RA * (A_LOADS * w + q) + a_row;               // row inside the tile
            int row = m0 + rl;
            if (RAGGED)
                row = row < M ? row : M - 1;
            pa0[q] = A + (int64_t)row * lda + ((a_slot ^ ((rl >> SH) & (CA - 1))) << 4);
        }
        int ncol = n0 + ((b_slot ^ fB(b_row)) << 4);                      // fB(RB*q + b_row) == fB(b_row)
        if (RAGGED)
            ncol = ncol + 16 <= N ? ncol : N - 16;
#pragma unroll
        for (int q = 0; q < B_LOADS; ++q)
            pb0[q] = B + (int64_t)(RB * (B_LOADS * w + q) + b_row) * ldb + ncol;
        auto issue = [&](int step) __attribute__((always_inline)) {
            uint8_t *st = smem + (step % STAGES) * STAGE;
#pragma unroll
            for (int q = 0; q < A_LOADS; ++q)
                __builtin_amdgcn_global_load_lds(
                    (const void __attribute__((address_space(1))) *)(pa0[q] + (int64_t)step * BKB),
                    (void __attribute__((address_space(3))) *)(st + (A_LOADS * w + q) * 1024), 16, 0, 0);
#pragma unroll
            for (int q = 0; q < B_LOADS; ++q)
                __builtin_amdgcn_global_load_lds(
                    (const void __attribute__((address_space(1))) *)(pb0[q] + (int64_t)step * BKB * ldb),
                    (void __attribute__((address_space(3))) *)(st + A_BYTES + (B_LOADS * w + q) * 1024), 16, 0, 0);
        };
        constexpr int AHEAD = STAGES - 1;
        for (int s = 0; s < AHEAD && s < nsteps; ++s)
            issue(s);
        int s = 0;
        for (; s + AHEAD < nsteps; ++s) {
            // the loads of steps s+1 .. s+AHEAD-1 may stay in flight; those of step s must have landed
            constexpr int vm = (AHEAD - 1) * LOADS;
            static_assert(vm < 64, "vmcnt is a 6-bit counter");
            __builtin_amdgcn_s_waitcnt((vm & 15) | ((vm >> 4) << 14) | 0x0f70);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            issue(s + AHEAD);
        }
        for (; s < nsteps; ++s) {
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): no further loads are issued
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (U8)
            asm volatile("s_barrier" ::: "memory");  // matches the consumers' barrier behind their byte sums
        return;
    }

    // ---------------------------------------------------------------------- consumers
    const int wm = wave & 1, wn = wave >> 1;
    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    // fragment addresses inside a stage for depth step ks = 0; the others follow by XOR / addition below
    const int l32 = lane & 31, khalf = lane >> 5;
    int a_row_off[TM], a_swz[TM], b_off[TN][2];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = (wm * TM + i) * 32 + l32;
        a_row_off[i] = row * BKB;
        a_swz[i] = (row >> SH) & (CA - 1);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int chunk = (wn * TN + j) * 2 + (l32 >> 4);  // 16-column chunk of the tile row
        const int jj = lane & 15;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int row = 16 * khalf + 8 * r + (jj >> 1);  // + 32*ks, which leaves fB(row) unchanged
            b_off[j][r] = A_BYTES + row * BN + ((chunk ^ fB(row)) << 4) + 8 * (jj & 1);
        }
    }
    auto read_frags = [&](int stage, int ks, v4i(&af)[TM], v4i(&bf)[TN]) __attribute__((always_inline)) {
        const uint8_t *st = smem + stage * STAGE;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            af[i] = *reinterpret_cast<const v4i *>(st + a_row_off[i] + (((2 * ks + khalf) ^ a_swz[i]) << 4));
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                (v2i __attribute__((address_space(3))) *)(st + b_off[j][0] + ks * 32 * BN));
            const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                (v2i __attribute__((address_space(3))) *)(st + b_off[j][1] + ks * 32 * BN));
            bf[j] = v4i{lo[0], lo[1], hi[0], hi[1]};
        }
    };
    // Unsigned operands: the fragments hold raw bytes.  Each is re-biased (XOR) right before its first MFMA, and one
    // wave per row block / column block adds the raw bytes up (v_sad_u8 against zero) for the corrections of eq. (3):
    // waves (0,0) and (1,1) sum the A rows of their row block, waves (1,0) and (0,1) the B columns of their column
    // block.  The main loop is instantiated once per role (no per-instruction selects), and the preparation of row
    // i+1 issues behind the MFMAs of row i.
    const bool sum_a = U8 && wm == wn, sum_b = U8 && wm != wn;
    uint32_t rs[TM], cs[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
        rs[i] = 0u;
#pragma unroll
    for (int j = 0; j < TN; ++j)
        cs[j] = 0u;
    auto flip = [&](v4i &f) __attribute__((always_inline)) {
        f = v4i{(int)((uint32_t)f[0] ^ FLIP), (int)((uint32_t)f[1] ^ FLIP), (int)((uint32_t)f[2] ^ FLIP), (int)((uint32_t)f[3] ^ FLIP)};
    };
    auto add_bytes = [&](const v4i &f, uint32_t &t) __attribute__((always_inline)) {
        t = bytesum((uint32_t)f[0], bytesum((uint32_t)f[1], bytesum((uint32_t)f[2], bytesum((uint32_t)f[3], t))));
    };
    // rows i0 .. i1-1 of the wave's 4 x 2 MFMA tiles; the B fragments are prepared with row 0
    auto mfma_rows = [&](auto sa, auto sb, v4i(&af)[TM], v4i(&bf)[TN], int i0, int i1) __attribute__((always_inline)) {
#pragma unroll
        for (int i = i0; i < i1; ++i) {
            if constexpr (U8) {
                if (i == 0) {
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        if constexpr (decltype(sb)::value)
                            add_bytes(bf[j], cs[j]);
                        flip(bf[j]);
                    }
                }
                if constexpr (decltype(sa)::value)
                    add_bytes(af[i], rs[i]);
                flip(af[i]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    };

    // Per MFMA depth step: the first two MFMAs, then the fragment reads of the next depth step, then the other six.
    // The compiler waits for ALL outstanding LDS reads before the first use of a fragment, so the reads of the next
    // depth step are issued only after the current fragments have been touched; six MFMAs (192 cycles) cover their
    // latency.  Two fragment sets alternate; the barrier sits in front of the last depth step of a stage, whose
    // fragments are in registers by then, so that the first fragments of the next stage can be read behind it.
    auto main_loop = [&](auto sa, auto sb) __attribute__((always_inline)) {
        v4i fa[2][TM], fb[2][TN];
        lds_barrier();  // barrier 0
        read_frags(0, 0, fa[0], fb[0]);
        int stage = 0;
        for (int s = 0; s + 1 < nsteps; ++s) {
            const int next = stage + 1 == STAGES ? 0 : stage + 1;
    #pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int cur = ks & 1;
                if (ks == KS - 1)
                    lds_barrier();  // barrier s+1; every read of step s has completed
                mfma_rows(sa, sb, fa[cur], fb[cur], 0, 1);
                __builtin_amdgcn_sched_barrier(0);
                if (ks == KS - 1)
                    read_frags(next, 0, fa[cur ^ 1], fb[cur ^ 1]);
                else
                    read_frags(stage, ks + 1, fa[cur ^ 1], fb[cur ^ 1]);
                __builtin_amdgcn_sched_barrier(0);
                mfma_rows(sa, sb, fa[cur], fb[cur], 1, TM);
                __builtin_amdgcn_sched_barrier(0);
            }
            stage = next;
        }
    #pragma unroll
        for (int ks = 0; ks < KS; ++ks) {  // last stage: nothing follows it
            const int cur = ks & 1;
            mfma_rows(sa, sb, fa[cur], fb[cur], 0, 1);
            __builtin_amdgcn_sched_barrier(0);
            if (ks + 1 < KS)
                read_frags(stage, ks + 1, fa[cur ^ 1], fb[cur ^ 1]);
            __builtin_amdgcn_sched_barrier(0);
            mfma_rows(sa, sb, fa[cur], fb[cur], 1, TM);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using std::false_type;
    using std::true_type;
    if (sum_a)
        main_loop(true_type{}, false_type{});
    else if (sum_b)
        main_loop(false_type{}, true_type{});
    else
        main_loop(false_type{}, false_type{});

    // U8: sums -> LDS, [index][depth half]; every row / column block has exactly one summing wave
    uint32_t *rsum = sums, *csum = sums + (U8 ? BM * 2 : 0);
    if constexpr (U8) {
        if (sum_a) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                rsum[((wm * TM + i) * 32 + l32) * 2 + khalf] = rs[i];
        }
        if (sum_b) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
                csum[((wn * TN + j) * 32 + l32) * 2 + khalf] = cs[j];
        }
        lds_barrier();
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int lcol = (wn * TN + j) * 32 + (lane & 31);
            const int col = n0 + lcol;
            int32_t ccorr = 0;
            if constexpr (U8)  // signed sums = unsigned sums - 128 per byte; all K bytes are real (whole tiles)
                ccorr = K * zA * zB - zA * ((int32_t)(csum[lcol * 2] + csum[lcol * 2 + 1]) - 128 * K);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lrow = (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                int32_t out = acc[i][j][r];
                if constexpr (U8)
                    out += ccorr - zB * ((int32_t)(rsum[lrow * 2] + rsum[lrow * 2 + 1]) - 128 * K);
                if (!RAGGED || (m0 + lrow < M && col < N))
                    C[(int64_t)(m0 + lrow) * ldc + col] = out;
            }
        }
}

}  // namespace

// How the 4-wave kernel fetches a problem with BM x BN tiles (see the fetch modes in gemm_i8_tile)
int i8_fetch_mode(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb, int BM, int BN)
{
    const bool aligned = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(B) % 4 == 0) && (ldb % 4 == 0);
    const bool whole = (M % BM) == 0 && (N % BN) == 0 && (K % BK) == 0;
    const bool can_clamp = (N % 4) == 0 && (K % 16) == 0 && N >= 4 && K >= 16;
    return (aligned && whole) ? 0 : (aligned && can_clamp) ? 1 : (N >= 4 && K >= BK) ? 2 : 3;
}

hipError_t launch_gemm_i8_group(const I8GroupHeader *table_dev, uint32_t count, uint32_t workgroups, hipStream_t stream)
{
    hipLaunchKernelGGL(gemm_i8_group_kernel, dim3(workgroups), dim3(256), 0, stream, table_dev, count);
    return hipGetLastError();
}

namespace {

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
    const int mode = i8_fetch_mode(M, N, K, A, lda, B, ldb, BM, BN);
    const dim3 g((unsigned)grid), b(256);
    if (mode == 0)
        hipLaunchKernelGGL((gemm_i8_mfma_kernel<TM, TN, 0, U8>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B,
                           ldb, C, ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    else if (mode == 1)
        hipLaunchKernelGGL((gemm_i8_mfma_kernel<TM, TN, 1, U8>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B,
                           ldb, C, ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    else if (mode == 2)
        hipLaunchKernelGGL((gemm_i8_mfma_kernel<TM, TN, 2, U8>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B,
                           ldb, C, ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    else
        hipLaunchKernelGGL((gemm_i8_mfma_kernel<TM, TN, 3, U8>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B,
                           ldb, C, ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    return hipGetLastError();
}

// Wave-specialised 256 x 128 instance; returns hipErrorNotSupported when the operands are not aligned or the shape
// needs byte-wise fetches (the caller then falls back to the 4-wave kernel).
template <bool U8, int DEPTH>
hipError_t launch_ws(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                     int32_t *C, int64_t ldc, hipStream_t stream, int zA, int zB)
{
    constexpr int BM = 256, BN = 128;
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
    const dim3 g((unsigned)grid), b(512);
    if (aligned && whole)
        hipLaunchKernelGGL((gemm_i8_ws_kernel<0, U8, DEPTH>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B, ldb, C,
                           ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    else if (aligned && can_clamp)
        hipLaunchKernelGGL((gemm_i8_ws_kernel<1, U8, DEPTH>), g, b, 0, stream, (int)M, (int)N, (int)K, A, lda, B, ldb, C,
                           ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

// Direct-to-LDS instances; hipErrorNotSupported unless every 16-byte chunk is aligned, the depth is a whole number
// of stages and (RAGGED = false) the tiles are whole.
template <int STAGES, int BKB, bool U8, int TM, int TN, bool RAGGED>
hipError_t launch_dl(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                     int32_t *C, int64_t ldc, hipStream_t stream, int zA, int zB)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    const bool ok = (K % BKB) == 0 && K >= BKB && (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 16 == 0) &&
                    (reinterpret_cast<uintptr_t>(B) % 16 == 0) && (ldb % 16 == 0) &&
                    (RAGGED ? ((N % 16) == 0 && N >= 16) : ((M % BM) == 0 && (N % BN) == 0));
    if (!ok)
        return hipErrorNotSupported;
    const int nMB = (int)((M + BM - 1) / BM), nNB = (int)((N + BN - 1) / BN);
    const int64_t tiles = (int64_t)nMB * nNB;
    const int tiles_per_xcd = (int)((tiles + 7) / 8);
    const int64_t grid = (int64_t)tiles_per_xcd * 8;
    if (grid > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((gemm_i8_dl_kernel<STAGES, BKB, U8, TM, TN, RAGGED>), dim3((unsigned)grid), dim3(512), 0, stream,
                       (int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, nMB, nNB, tiles_per_xcd, zA, zB);
    return hipGetLastError();
}

// One tile shape of the direct-to-LDS kernel: depth stages of 128 bytes when the depth allows, else 64; the 256 x 128
// tile has an instance without edge handling for whole tiles.
template <bool U8, int TM, int TN>
hipError_t launch_dl_tile(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                          int32_t *C, int64_t ldc, hipStream_t stream, int zA, int zB)
{
    const bool whole = TM == 4 && (M % (64 * TM)) == 0 && (N % (64 * TN)) == 0;
    if (K % 128 == 0)
        return whole ? launch_dl<3, 128, U8, TM, TN, TM != 4>(M, N, K, A, lda, B, ldb, C, ldc, stream, zA, zB)
                     : launch_dl<3, 128, U8, TM, TN, true>(M, N, K, A, lda, B, ldb, C, ldc, stream, zA, zB);
    return whole ? launch_dl<4, 64, U8, TM, TN, TM != 4>(M, N, K, A, lda, B, ldb, C, ldc, stream, zA, zB)
                 : launch_dl<4, 64, U8, TM, TN, true>(M, N, K, A, lda, B, ldb, C, ldc, stream, zA, zB);
}

// Shape-based choice among the direct-to-LDS instances.  A tile shape is eligible if it yields enough workgroups
// (256 x 128: half a machine of them; 128 x 128: about 112; 64 x 64: always - small problems are latency-bound and more,
// smaller workgroups win); among the eligible ones the cheapest wins, cost = multiply-adds including those of the
// padding rows and columns of ragged tiles, divided by the rate the shape reaches on large problems relative to
// 256 x 128 (measured: 0.8 and 0.47).  Thresholds and rates come from sweeps over conv-shaped problems.
template <bool U8>
hipError_t launch_dl_auto(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                          int32_t *C, int64_t ldc, hipStream_t stream, int zA, int zB)
{
    const int64_t m256 = (M + 255) / 256, m128 = (M + 127) / 128, m64 = (M + 63) / 64;
    const int64_t n128 = (N + 127) / 128, n64 = (N + 63) / 64;
    const double c256 = m256 * n128 >= 128 ? (double)(m256 * 256) * (double)(n128 * 128) : 1e300;
    const double c128 = m128 * n128 >= 112 ? (double)(m128 * 128) * (double)(n128 * 128) / 0.8 : 1e300;
    const double c64 = (double)(m64 * 64) * (double)(n64 * 64) / 0.47;
    if (c256 <= c128 && c256 <= c64)
        return launch_dl_tile<U8, 4, 2>(M, N, K, A, lda, B, ldb, C, ldc, stream, zA, zB);
    if (c128 <= c64)
        return launch_dl_tile<U8, 2, 2>(M, N, K, A, lda, B, ldb, C, ldc, stream, zA, zB);
    return launch_dl_tile<U8, 1, 1>(M, N, K, A, lda, B, ldb, C, ldc, stream, zA, zB);
}

std::atomic<int> g_i8_forced{-1};  // benchmark hook; read once per call

}  // namespace

void i8_force_tile(int t) { g_i8_forced.store(t, std::memory_order_relaxed); }

hipError_t launch_gemm_i8(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                          int32_t *C, int64_t ldc, hipStream_t stream)
{
    const int64_t tiles = ((M + 255) / 256) * ((N + 127) / 128);
    const int forced = g_i8_forced.load(std::memory_order_relaxed);
    int t = forced;
    // a right operand of at most 16 columns would leave a matrix-core tile almost empty: stream A with dot products
    if (t < 0 && N <= 16 && M >= 64)
        return launch_gemm_i8_skinny(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (t < 0) {
        // direct-to-LDS instances wherever alignment and depth allow, then the register-staged ones
        const hipError_t e = launch_dl_auto<false>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
        if (e != hipErrorNotSupported)
            return e;
        t = tiles >= 128 ? 3 : 0;
    }
    if (t >= 6) {
        const hipError_t e = t == 6   ? launch_dl<4, 64, false, 4, 2, true>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0)
                             : t == 7 ? launch_dl_tile<false, 4, 2>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0)
                             : t == 8 ? launch_dl_tile<false, 2, 2>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0)
                                      : launch_dl_tile<false, 1, 1>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
        if (e != hipErrorNotSupported)
            return e;
        t = 3;
    }
    if (t >= 3) {
        const hipError_t e = t == 3   ? launch_ws<false, 3>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0)
                             : t == 4 ? launch_ws<false, 2>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0)
                                      : launch_ws<false, 4>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
        if (e != hipErrorNotSupported)
            return e;
        t = 2;
    }
    if (t == 1)
        return launch_tile<4, 4, false>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
    if (t == 2)
        return launch_tile<4, 2, false>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
    // unforced small problems: 64 x 64 tiles put four times as many workgroups on the machine
    if (forced < 0 && ((M + 127) / 128) * ((N + 127) / 128) < 128)
        return launch_tile<1, 1, false>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
    return launch_tile<2, 2, false>(M, N, K, A, lda, B, ldb, C, ldc, stream, 0, 0);
}

// unsigned operands with zero points; zA, zB in [0, 255]
hipError_t launch_gemm_u8(int64_t M, int64_t N, int64_t K, const uint8_t *A, int64_t lda, const uint8_t *B, int64_t ldb,
                          int zA, int zB, int32_t *C, int64_t ldc, hipStream_t stream)
{
    const int64_t tiles = ((M + 255) / 256) * ((N + 127) / 128);
    const int8_t *a = reinterpret_cast<const int8_t *>(A), *b = reinterpret_cast<const int8_t *>(B);
    hipError_t e = launch_dl_auto<true>(M, N, K, a, lda, b, ldb, C, ldc, stream, zA - 128, zB - 128);
    if (e != hipErrorNotSupported)
        return e;
    if (tiles >= 128) {
        e = launch_ws<true, 3>(M, N, K, a, lda, b, ldb, C, ldc, stream, zA - 128, zB - 128);
        if (e != hipErrorNotSupported)
            return e;
        return launch_tile<4, 2, true>(M, N, K, a, lda, b, ldb, C, ldc, stream, zA - 128, zB - 128);
    }
    if (((M + 127) / 128) * ((N + 127) / 128) < 128)
        return launch_tile<1, 1, true>(M, N, K, a, lda, b, ldb, C, ldc, stream, zA - 128, zB - 128);
    return launch_tile<2, 2, true>(M, N, K, a, lda, b, ldb, C, ldc, stream, zA - 128, zB - 128);
}

}  // namespace lowbit
