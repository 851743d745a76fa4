// Skinny popcount GEMM (fully connected layers, small batch): one operand has only a few bit strings.
//
// The products are those of eq. (6) / (7) of the paper, evaluated in the same reduced forms as the tiled kernels
// (see gemm_popc.hip).  What differs is the decomposition, because the work is bound by streaming the large
// operand ("X", rowsX bit strings) from HBM exactly once:
//   * the small operand ("Y", NS = 8, 16 or 32 bit strings per workgroup column block: the smallest that holds all
//     of them, so that X is streamed once) is staged in LDS,
//     converted to (nz, neg) planes when ternary;
//   * a wave owns R strings of X and its 64 lanes split the depth: lane l takes depth words l, l+64, ... of the
//     current chunk, so every load instruction of a wave reads one contiguous kilobyte of X;
//   * each lane accumulates R x NS partial products over its depth slice in registers; at the end the wave
//     reduces them across lanes with a halving butterfly (R*NS values shrink to one per lane pair) and
//     writes int32 C.
// Kinds: BNN (X, Y binary), TNN (X, Y ternary), TBN (X ternary, Y binary), TBN_SV (X binary, Y ternary: gemm_tbn
// with few ternary rows; the non-zero counts of the Y strings are taken while they are staged and summed in LDS).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

// NS strings of Y per workgroup; KC depth words per LDS chunk (JW per lane), smaller for more strings so that the
// chunk stays within 64 KB of LDS
template <int NS> struct SkChunk { static constexpr int KC = NS <= 8 ? 256 : NS == 16 ? 256 : 128; };

__device__ __forceinline__ uint32_t and_vv(uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_and_b32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t xor_vv(uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_xor_b32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// (a ^ b) & m
__device__ __forceinline__ uint32_t xor_and_vvv(uint32_t a, uint32_t b, uint32_t m)
{
    uint32_t r;
    asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x28" : "=v"(r) : "v"(a), "v"(b), "v"(m));
    return r;
}
__device__ __forceinline__ void popc_acc(int32_t &acc, uint32_t x)
{
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
}

template <int KIND> struct SkTraits;
template <> struct SkTraits<KIND_BNN> { using X = uint2; using Y = uint2; static constexpr int ACC = 1; };
template <> struct SkTraits<KIND_TNN> { using X = uint4; using Y = uint4; static constexpr int ACC = 2; };
template <> struct SkTraits<KIND_TBN> { using X = uint4; using Y = uint2; static constexpr int ACC = 1; };
template <> struct SkTraits<KIND_TBN_SV> { using X = uint2; using Y = uint4; static constexpr int ACC = 1; };

__device__ __forceinline__ uint2 zero2() { return make_uint2(0u, 0u); }
__device__ __forceinline__ uint4 zero4() { return make_uint4(0u, 0u, 0u, 0u); }
template <typename T> __device__ __forceinline__ T zero_entry();
template <> __device__ __forceinline__ uint2 zero_entry<uint2>() { return zero2(); }
template <> __device__ __forceinline__ uint4 zero_entry<uint4>() { return zero4(); }
__device__ __forceinline__ uint4 nz_neg(uint4 e) { return make_uint4(e.x | e.z, e.y | e.w, e.z, e.w); }
__device__ __forceinline__ uint2 nz_neg(uint2 e) { return e; }

// Sum val[0..CNT) over the lanes that differ in bit BIT and below; afterwards val[0] of lane l holds the total of
// the value whose index is formed by the lane bits consumed while CNT > 1 (most significant first).
template <int CNT, int BIT> __device__ __forceinline__ void reduce_halving(int32_t *val, int lane)
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
            reduce_halving<HALF, BIT / 2>(val, lane);
        } else {
            val[0] += __shfl_xor(val[0], BIT, 64);
            reduce_halving<1, BIT / 2>(val, lane);
        }
    }
}

template <int KIND, int R, int WAVES, bool TR, int NS = 8>
__global__ __launch_bounds__(64 * WAVES) void gemm_skinny_kernel(const void *__restrict__ Xp_, const void *__restrict__ Yp_,
                                                          int rowsX, int rowsY, int KW, int K,
                                                          int32_t *__restrict__ C, int64_t ldc, int c16)
{
    using T = SkTraits<KIND>;
    using XE = typename T::X;
    using YE = typename T::Y;
    constexpr int KC = SkChunk<NS>::KC, JW = KC / 64;
    constexpr int V = R * NS;  // partial sums per lane
    static_assert((V & (V - 1)) == 0 && V <= 64 && V >= 2, "R*NS must be a power of two <= 64");

    __shared__ YE ylds[NS][KC];
    __shared__ int32_t ynnz[NS];  // TBN_SV: non-zero positions of each Y string

    const XE *__restrict__ Xp = static_cast<const XE *>(Xp_);
    const YE *__restrict__ Yp = static_cast<const YE *>(Yp_);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int x0 = (blockIdx.x * WAVES + wave) * R;
    const int y0 = blockIdx.y * NS;

    const XE *xrow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int xr = x0 + r;
        xr = xr < rowsX ? xr : rowsX - 1;
        xrow[r] = Xp + (int64_t)xr * KW;
    }

    int32_t acc[T::ACC][R][NS];
#pragma unroll
    for (int a = 0; a < T::ACC; ++a)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int n = 0; n < NS; ++n)
                acc[a][r][n] = 0;
    int32_t nnz[R];
#pragma unroll
    for (int r = 0; r < R; ++r)
        nnz[r] = 0;
    if constexpr (KIND == KIND_TBN_SV) {
        if (tid < NS)
            ynnz[tid] = 0;
        __syncthreads();
    }

    for (int kc = 0; kc < KW; kc += KC) {
        // Y loads are issued first (clamped addresses, no branches)
        constexpr int NT = 64 * WAVES;
        constexpr int YPT = (NS * KC + NT - 1) / NT;
        YE ypre[YPT];
#pragma unroll
        for (int i = 0; i < YPT; ++i) {
            const int e = tid + i * NT;
            const int n = e / KC, g = e % KC;
            const bool ok = (e < NS * KC) && (y0 + n < rowsY) && (kc + g < KW);
            const int yn = ok ? y0 + n : rowsY - 1;
            const int yg = ok ? kc + g : KW - 1;
            const YE y = Yp[(int64_t)yn * KW + yg];
            ypre[i] = ok ? y : zero_entry<YE>();
        }
        // then the X loads, the long-latency HBM stream; the Y data (L2 hits) returns first and is staged while
        // X is still in flight
        XE xa[R][JW];
#pragma unroll
        for (int j = 0; j < JW; ++j) {
            const int g = kc + j * 64 + lane;
#pragma unroll
            for (int r = 0; r < R; ++r)
            {
                const XE x = xrow[r][g < KW ? g : KW - 1];
                xa[r][j] = g < KW ? x : zero_entry<XE>();
            }
        }
        if (kc)
            __syncthreads();  // previous chunk fully consumed
#pragma unroll
        for (int i = 0; i < YPT; ++i) {
            const int e = tid + i * NT;
            if (NS * KC % NT == 0 || e < NS * KC) {
                const YE y = nz_neg(ypre[i]);
                ylds[e / KC][e % KC] = y;
                if constexpr (KIND == KIND_TBN_SV) {
                    const int cnt = __builtin_popcount(y.x) + __builtin_popcount(y.y);
                    if (cnt)
                        atomicAdd(&ynnz[e / KC], cnt);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < JW; ++j) {
            XE x[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                x[r] = nz_neg(xa[r][j]);
                if constexpr (KIND == KIND_TBN) {
                    popc_acc(nnz[r], x[r].x);
                    popc_acc(nnz[r], x[r].y);
                }
            }
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const YE y = ylds[n][j * 64 + lane];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if constexpr (KIND == KIND_BNN) {
                        popc_acc(acc[0][r][n], xor_vv(x[r].x, y.x));
                        popc_acc(acc[0][r][n], xor_vv(x[r].y, y.y));
                    } else if constexpr (KIND == KIND_TNN) {
                        const uint32_t m0 = and_vv(x[r].x, y.x), m1 = and_vv(x[r].y, y.y);
                        const uint32_t u0 = xor_and_vvv(x[r].z, y.z, m0), u1 = xor_and_vvv(x[r].w, y.w, m1);
                        popc_acc(acc[0][r][n], m0);
                        popc_acc(acc[1][r][n], u0);
                        popc_acc(acc[0][r][n], m1);
                        popc_acc(acc[1][r][n], u1);
                    } else if constexpr (KIND == KIND_TBN) {
                        popc_acc(acc[0][r][n], xor_and_vvv(x[r].z, y.x, x[r].x));
                        popc_acc(acc[0][r][n], xor_and_vvv(x[r].w, y.y, x[r].y));
                    } else {
                        popc_acc(acc[0][r][n], xor_and_vvv(y.z, x[r].x, y.x));
                        popc_acc(acc[0][r][n], xor_and_vvv(y.w, x[r].y, y.y));
                    }
                }
            }
        }
    }

    // per-lane partial results; BNN's "K - 2*popcount" is applied after the reduction
    int32_t val[V];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int n = 0; n < NS; ++n) {
            if constexpr (KIND == KIND_BNN || KIND == KIND_TBN_SV)
                val[r * NS + n] = acc[0][r][n];
            else if constexpr (KIND == KIND_TNN)
                val[r * NS + n] = acc[0][r][n] - 2 * acc[1][r][n];
            else
                val[r * NS + n] = nnz[r] - 2 * acc[0][r][n];
        }

    // halving butterfly: at lane-bit b the lanes with the bit set keep the upper half of the values
    reduce_halving<V, 32>(val, lane);
    // lane l now holds the total of value index (l >> (6 - log2 V)); one lane of each group stores it
    constexpr int GROUP = 64 / V;
    if ((lane % GROUP) == 0) {
        const int idx = lane / GROUP;
        const int r = idx / NS, n = idx % NS;
        const int xr = x0 + r, yn = y0 + n;
        if (xr < rowsX && yn < rowsY) {
            int32_t out = val[0];
            if constexpr (KIND == KIND_BNN)
                out = K - 2 * out;
            if constexpr (KIND == KIND_TBN_SV)
                out = ynnz[n] - 2 * out;  // complete: the last staging was followed by a barrier
            const int64_t at = TR ? (int64_t)yn * ldc + xr : (int64_t)xr * ldc + yn;
            if (c16)
                reinterpret_cast<int16_t *>(C)[at] = (int16_t)out;  // K <= 32767 checked on the host
            else
                C[at] = out;
        }
    }
}

template <int KIND, int R, int WAVES, bool TR, int NS = 8> hipError_t launch_sk(const SkinnyArgs &a)
{
    const int64_t gx = ((int64_t)a.rowsX + WAVES * R - 1) / (WAVES * R);
    const int64_t gy = ((int64_t)a.rowsY + NS - 1) / NS;
    if (gx > 0x7fffffffLL || gy > 65535)
        return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((gemm_skinny_kernel<KIND, R, WAVES, TR, NS>), dim3((unsigned)gx, (unsigned)gy), dim3(64 * WAVES),
                       0, a.stream, a.Xp, a.Yp, a.rowsX, a.rowsY, a.KW, a.K, a.C, a.ldc, a.c16);
    return hipGetLastError();
}

std::atomic<int> g_skinny_forced{-1};  // benchmark hook; read once per call

template <int KIND> hipError_t launch_kind(const SkinnyArgs &a, bool tr)
{
    // (rows per wave, waves per workgroup), measured on M x 4096 .. 65536 x 1 .. 16 problems: large row counts
    // stream best with 2 rows per wave (binary operands, half the bytes per row: 4); a few thousand rows are
    // latency-bound and want many small waves in flight
    int cfg = g_skinny_forced.load(std::memory_order_relaxed);
    if (cfg < 0) {
        if (a.rowsX >= 16384)
            cfg = (KIND == KIND_BNN || KIND == KIND_TBN_SV) ? 7 : KIND == KIND_TNN ? 3 : 1;
        else if (a.rowsX >= 6144)
            cfg = 3;
        else if (a.rowsX >= 2048)
            cfg = 5;
        else
            cfg = 2;
        if (a.rowsY > 16 && a.rowsX >= 2048)
            cfg = 3;  // 32 strings per workgroup: 2 rows per wave halve the LDS reads per product
    }
    // more than 8 short strings: 16 or 32 per workgroup (the long operand is still streamed once), with the
    // configurations whose R x NS partial sums fit a lane
    if (a.rowsY > 8) {
        const bool wide = a.rowsY > 16;
#define LB_SK_NS(R, W)                                                                                          \
    (wide ? (tr ? launch_sk<KIND, R, W, true, 32>(a) : launch_sk<KIND, R, W, false, 32>(a))                    \
          : (tr ? launch_sk<KIND, R, W, true, 16>(a) : launch_sk<KIND, R, W, false, 16>(a)))
        switch (cfg) {
        case 1: return LB_SK_NS(2, 4);
        case 0:
        case 3:
        case 6:
        case 7: return LB_SK_NS(2, 8);
        default: return LB_SK_NS(1, 8);  // 16 waves of 1 row would spill: 32 x 2 accumulators at 128 registers
        }
#undef LB_SK_NS
    }
    switch (cfg) {
    case 0: return tr ? launch_sk<KIND, 4, 4, true>(a) : launch_sk<KIND, 4, 4, false>(a);
    case 1: return tr ? launch_sk<KIND, 2, 4, true>(a) : launch_sk<KIND, 2, 4, false>(a);
    case 2: return tr ? launch_sk<KIND, 1, 4, true>(a) : launch_sk<KIND, 1, 4, false>(a);
    case 3: return tr ? launch_sk<KIND, 2, 8, true>(a) : launch_sk<KIND, 2, 8, false>(a);
    case 4: return tr ? launch_sk<KIND, 1, 16, true>(a) : launch_sk<KIND, 1, 16, false>(a);
    case 5: return tr ? launch_sk<KIND, 1, 8, true>(a) : launch_sk<KIND, 1, 8, false>(a);
    case 6: return tr ? launch_sk<KIND, 2, 16, true>(a) : launch_sk<KIND, 2, 16, false>(a);
    default: return tr ? launch_sk<KIND, 4, 8, true>(a) : launch_sk<KIND, 4, 8, false>(a);
    }
}

}  // namespace

int skinny_num_configs() { return 8; }
void skinny_force_config(int cfg) { g_skinny_forced.store(cfg, std::memory_order_relaxed); }
int skinny_forced_config() { return g_skinny_forced.load(std::memory_order_relaxed); }

hipError_t launch_gemm_skinny(int kind, const SkinnyArgs &a, bool transposed)
{
    switch (kind) {
    case KIND_BNN: return launch_kind<KIND_BNN>(a, transposed);
    case KIND_TNN: return launch_kind<KIND_TNN>(a, transposed);
    case KIND_TBN: return launch_kind<KIND_TBN>(a, transposed);
    case KIND_TBN_SV: return launch_kind<KIND_TBN_SV>(a, transposed);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lowbit
