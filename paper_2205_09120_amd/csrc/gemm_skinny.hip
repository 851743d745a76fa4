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

// Value of v held by lane (l ^ BIT).  Within a half of the wave (BIT < 32) one LDS-pipe swizzle with an immediate
// pattern, no address arithmetic; across the halves a permute through the byte address of lane l ^ 32 (swap32, computed
// once per kernel).
template <int BIT> __device__ __forceinline__ int32_t lane_xor(int32_t v, int swap32)
{
    if constexpr (BIT == 32)
        return __builtin_amdgcn_ds_bpermute(swap32, v);
    else
        return __builtin_amdgcn_ds_swizzle(v, (BIT << 10) | 0x1f);  // bit-mask mode: and 0x1f, or 0, xor BIT
}

// Sum val[0..CNT) over the lanes that differ in bit BIT and below; afterwards val[0] of lane l holds the total of
// the value whose index is formed by the lane bits consumed while CNT > 1 (most significant first).
template <int CNT, int BIT> __device__ __forceinline__ void reduce_halving(int32_t *val, int lane, int swap32)
{
    if constexpr (BIT >= 1) {
        if constexpr (CNT > 1) {
            constexpr int HALF = CNT / 2;
            const bool upper = (lane & BIT) != 0;
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                const int32_t send = upper ? val[i] : val[i + HALF];
                const int32_t keep = upper ? val[i + HALF] : val[i];
                val[i] = keep + lane_xor<BIT>(send, swap32);
            }
            reduce_halving<HALF, BIT / 2>(val, lane, swap32);
        } else {
            val[0] += lane_xor<BIT>(val[0], swap32);
            reduce_halving<1, BIT / 2>(val, lane, swap32);
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
    reduce_halving<V, 32>(val, lane, (lane ^ 32) << 2);
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

// One 64-bit depth word of X against the same word of Y, added to the partial sums of one (row, string) pair.
// x and y hold (nz, neg) planes when ternary (two dwords per plane) and the sign bits when binary.
template <int KIND, typename XW, typename YW>
__device__ __forceinline__ void sk_mac(int32_t &a0, int32_t &a1, const XW &x, const YW &y)
{
    if constexpr (KIND == KIND_BNN) {
        popc_acc(a0, xor_vv(x.x, y.x));
        popc_acc(a0, xor_vv(x.y, y.y));
    } else if constexpr (KIND == KIND_TNN) {
        const uint32_t m0 = and_vv(x.x, y.x), m1 = and_vv(x.y, y.y);
        const uint32_t u0 = xor_and_vvv(x.z, y.z, m0), u1 = xor_and_vvv(x.w, y.w, m1);
        popc_acc(a0, m0);
        popc_acc(a1, u0);
        popc_acc(a0, m1);
        popc_acc(a1, u1);
    } else if constexpr (KIND == KIND_TBN) {
        popc_acc(a0, xor_and_vvv(x.z, y.x, x.x));
        popc_acc(a0, xor_and_vvv(x.w, y.y, x.y));
    } else {
        popc_acc(a0, xor_and_vvv(y.z, x.x, y.x));
        popc_acc(a0, xor_and_vvv(y.w, x.y, y.y));
    }
}

// Streaming variant for at most NS short strings whose whole depth fits in LDS: Y is staged ONCE per workgroup, the
// grid is at most two workgroups per compute unit, and every wave walks over its row groups (R rows each) with a ring
// of D lane-steps of X in flight -- the loads of step s + D are issued right after step s has been multiplied, so the
// HBM stream never waits for a barrier or for the cross-lane reduction of a finished row.  A lane-step is one 16-byte
// load per lane and row: one depth word of a ternary string, two of a binary one (W), i.e. SW = 64 * W depth words per
// wave and step; a row has JWn = ceil(KW / SW) steps and the ring runs on across row boundaries.  Every wave that has
// work must have at least D steps.  The last round of Y loads is issued
// BEFORE the first X loads and waited for with those still in flight, so a short stream (one row per wave: the
// batch-8 fully connected layer) multiplies its first words while the rest of the row is still arriving.
// LDS layout of Y: entry (step jb, string n, word w of the step) at ((jb * NS + n) * SW + slot(w)); slot(w) = w, except
// for ternary Y next to binary X, where the two words a lane needs are 64 entries apart (conflict-free 16-byte reads).
template <int KIND, int R, int WAVES, bool TR, int NS, bool KFULL, int D>
__global__ __launch_bounds__(64 * WAVES) void gemm_skinny_stream_kernel(const void *__restrict__ Xp_,
                                                                        const void *__restrict__ Yp_, int rowsX,
                                                                        int rowsY, int KW, int K,
                                                                        int32_t *__restrict__ C, int64_t ldc, int c16,
                                                                        int JWn, int groups)
{
    using T = SkTraits<KIND>;
    using YE = typename T::Y;
    constexpr bool XBIN = sizeof(typename T::X) == 8;
    constexpr bool YTER = sizeof(YE) == 16;
    constexpr int W = XBIN ? 2 : 1;
    constexpr int SW = 64 * W;
    constexpr int NT = 64 * WAVES;
    constexpr int V = R * NS;
    constexpr int YU = 4;  // Y entries a thread stages per round
    static_assert((V & (V - 1)) == 0 && V <= 64 && V >= 2, "R*NS must be a power of two <= 64");
    static_assert((NS & (NS - 1)) == 0, "NS must be a power of two");

    extern __shared__ uint4 sk_smem[];
    YE *ylds = reinterpret_cast<YE *>(sk_smem);
    const int entries = JWn * NS * SW;
    int32_t *ynnz = reinterpret_cast<int32_t *>(ylds + entries);  // TBN_SV: non-zero positions of each Y string

    const YE *__restrict__ Yp = static_cast<const YE *>(Yp_);
    const uint4 *__restrict__ Xq = static_cast<const uint4 *>(Xp_);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int y0 = blockIdx.y * NS;
    const int rstride = XBIN ? KW / 2 : KW;  // 16-byte pieces per X string (binary: KW is even)

    if constexpr (KIND == KIND_TBN_SV) {
        if (tid < NS)
            ynnz[tid] = 0;
        __syncthreads();
    }

    // ---- Y staging: clamped addresses and masks instead of branches, so that the loads are unconditional
    YE yv[YU];
    uint32_t ym[YU];
    auto y_load = [&](int round) {
#pragma unroll
        for (int i = 0; i < YU; ++i) {
            const int e = (round * YU + i) * NT + tid;
            const int w = e & (SW - 1), t = e / SW;
            const int n = t & (NS - 1), jb = t / NS;
            const int slot = (W == 2 && YTER) ? (w & 63) * 2 + (w >> 6) : w;  // inverse of the layout rule
            const int g = jb * SW + slot;
            const bool ok = e < entries && y0 + n < rowsY && g < KW;
            yv[i] = Yp[(int64_t)(ok ? y0 + n : y0) * KW + (ok ? g : 0)];
            ym[i] = ok ? 0xffffffffu : 0u;
        }
    };
    auto y_store = [&](int round) {
#pragma unroll
        for (int i = 0; i < YU; ++i) {
            const int e = (round * YU + i) * NT + tid;
            YE y = yv[i];
            y.x &= ym[i];
            y.y &= ym[i];
            if constexpr (YTER) {
                y.z &= ym[i];
                y.w &= ym[i];
            }
            y = nz_neg(y);
            if (e < entries) {
                ylds[e] = y;
                if constexpr (KIND == KIND_TBN_SV) {
                    const int cnt = __builtin_popcount(y.x) + __builtin_popcount(y.y);
                    if (cnt)
                        atomicAdd(&ynnz[(e / SW) & (NS - 1)], cnt);
                }
            }
        }
    };

    // ---- X stream of this wave: row groups gw, gw + GW, ... ; loads and multiplications keep their own positions
    const int gw = blockIdx.x * WAVES + wave, GW = gridDim.x * WAVES;
    const int my_iters = gw < groups ? (groups - gw + GW - 1) / GW : 0;
    int lgroup = gw < groups ? gw : groups - 1, lj = 0;
    const uint4 *lx[R];
    auto set_rows = [&]() {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            int row = lgroup * R + r;
            row = row < rowsX ? row : rowsX - 1;
            lx[r] = Xq + (int64_t)row * rstride;
        }
    };
    set_rows();
    uint4 ring[D][R];
    auto issue = [&](int d) __attribute__((always_inline)) {
        int idx = lj * 64 + lane;
        if constexpr (!KFULL)
            idx = idx < rstride ? idx : rstride - 1;
#pragma unroll
        for (int r = 0; r < R; ++r)
            ring[d][r] = lx[r][idx];
        if (++lj == JWn) {
            lj = 0;
            lgroup += GW;
            lgroup = lgroup < groups ? lgroup : groups - 1;
            set_rows();
        }
    };

    const int rounds = (entries + NT * YU - 1) / (NT * YU);
    // whole problem (all NS strings, depth a multiple of the step, whole rounds): no clamps, no masks
    const bool y_whole = KFULL && rowsY - y0 >= NS && entries % (NT * YU) == 0;
    auto y_load_whole = [&](int round) {
#pragma unroll
        for (int i = 0; i < YU; ++i) {
            const int e = (round * YU + i) * NT + tid;
            const int w = e & (SW - 1), t = e / SW;
            const int n = t & (NS - 1), jb = t / NS;
            const int slot = (W == 2 && YTER) ? (w & 63) * 2 + (w >> 6) : w;
            yv[i] = Yp[(int64_t)(y0 + n) * KW + jb * SW + slot];
        }
    };
    auto y_store_whole = [&](int round) {
#pragma unroll
        for (int i = 0; i < YU; ++i) {
            const int e = (round * YU + i) * NT + tid;
            const YE y = nz_neg(yv[i]);
            ylds[e] = y;
            if constexpr (KIND == KIND_TBN_SV) {
                const int cnt = __builtin_popcount(y.x) + __builtin_popcount(y.y);
                if (cnt)
                    atomicAdd(&ynnz[(e / SW) & (NS - 1)], cnt);
            }
        }
    };
    if (y_whole) {
        for (int round = 0; round + 1 < rounds; ++round) {
            y_load_whole(round);
            y_store_whole(round);
        }
        y_load_whole(rounds - 1);
#pragma unroll
        for (int d = 0; d < D; ++d)
            issue(d);
        y_store_whole(rounds - 1);
    } else {
        for (int round = 0; round + 1 < rounds; ++round) {
            y_load(round);
            y_store(round);
        }
        y_load(rounds - 1);
#pragma unroll
        for (int d = 0; d < D; ++d)
            issue(d);
        y_store(rounds - 1);
    }
    __syncthreads();

    const int swap32 = (lane ^ 32) << 2;  // byte address of the partner lane in the other half of the wave
    int32_t acc[T::ACC][R][NS];
    int32_t nnz[R];
    auto clear = [&]() {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            nnz[r] = 0;
#pragma unroll
            for (int a = 0; a < T::ACC; ++a)
#pragma unroll
                for (int n = 0; n < NS; ++n)
                    acc[a][r][n] = 0;
        }
    };
    clear();
    int cgroup = gw, cj = 0;

    auto finish = [&]() __attribute__((always_inline)) {
        int32_t val[V];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                if constexpr (KIND == KIND_BNN || KIND == KIND_TBN_SV)
                    val[r * NS + n] = acc[0][r][n];
                else if constexpr (KIND == KIND_TNN)
                    val[r * NS + n] = acc[0][r][n] - 2 * acc[T::ACC - 1][r][n];
                else
                    val[r * NS + n] = nnz[r] - 2 * acc[0][r][n];
            }
        reduce_halving<V, 32>(val, lane, swap32);
        constexpr int GROUP = 64 / V;
        if ((lane % GROUP) == 0) {
            const int idx = lane / GROUP;
            const int r = idx / NS, n = idx % NS;
            const int xr = cgroup * R + r, yn = y0 + n;
            if (xr < rowsX && yn < rowsY) {
                int32_t out = val[0];
                if constexpr (KIND == KIND_BNN)
                    out = K - 2 * out;
                if constexpr (KIND == KIND_TBN_SV)
                    out = ynnz[n] - 2 * out;
                const int64_t at = TR ? (int64_t)yn * ldc + xr : (int64_t)xr * ldc + yn;
                if (c16)
                    reinterpret_cast<int16_t *>(C)[at] = (int16_t)out;  // K <= 32767 checked on the host
                else
                    C[at] = out;
            }
        }
    };

    // one step: take slot d of the ring, refill it at once (so that D loads stay in flight while this step is
    // multiplied), multiply
    auto consume = [&](int d, bool refill) __attribute__((always_inline)) {
        uint4 xv[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            xv[r] = ring[d][r];
        if (refill)
            issue(d);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if constexpr (!KFULL) {
                const uint32_t live = (cj * 64 + lane) < rstride ? 0xffffffffu : 0u;
                xv[r].x &= live;
                xv[r].y &= live;
                xv[r].z &= live;
                xv[r].w &= live;
            }
            if constexpr (!XBIN) {
                xv[r] = nz_neg(xv[r]);
                if constexpr (KIND == KIND_TBN) {
                    popc_acc(nnz[r], xv[r].x);
                    popc_acc(nnz[r], xv[r].y);
                }
            }
        }
        const YE *yb = ylds + (cj * NS) * SW;
#pragma unroll
        for (int n = 0; n < NS; ++n) {
            if constexpr (!XBIN) {
                const YE y = yb[n * SW + lane];
#pragma unroll
                for (int r = 0; r < R; ++r)
                    sk_mac<KIND>(acc[0][r][n], acc[T::ACC - 1][r][n], xv[r], y);
            } else if constexpr (!YTER) {
                // binary X, binary Y: the two words of the lane are adjacent in LDS
                const uint4 yy = *reinterpret_cast<const uint4 *>(yb + n * SW + lane * 2);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    sk_mac<KIND>(acc[0][r][n], acc[0][r][n], make_uint2(xv[r].x, xv[r].y), make_uint2(yy.x, yy.y));
                    sk_mac<KIND>(acc[0][r][n], acc[0][r][n], make_uint2(xv[r].z, xv[r].w), make_uint2(yy.z, yy.w));
                }
            } else {
                const YE ya = yb[n * SW + lane], yc = yb[n * SW + 64 + lane];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    sk_mac<KIND>(acc[0][r][n], acc[0][r][n], make_uint2(xv[r].x, xv[r].y), ya);
                    sk_mac<KIND>(acc[0][r][n], acc[0][r][n], make_uint2(xv[r].z, xv[r].w), yc);
                }
            }
        }
        if (++cj == JWn) {
            finish();
            clear();
            cj = 0;
            cgroup += GW;
        }
    };

    // nsteps >= D for every wave that has work (the launcher picks D accordingly).  The steady loop refills
    // unconditionally; the last D .. 2D-1 steps are peeled so that no load is issued beyond the wave's stream.
    if (my_iters > 0) {
        const int nsteps = my_iters * JWn;
        const int nfull = (nsteps - D) / D;
        for (int b = 0; b < nfull; ++b) {
#pragma unroll
            for (int d = 0; d < D; ++d)
                consume(d, true);
        }
        const int rest = nsteps - D - nfull * D;  // steps not yet issued: 0 .. D-1
#pragma unroll
        for (int d = 0; d < D; ++d)
            consume(d, d < rest);
#pragma unroll
        for (int d = 0; d < D - 1; ++d)
            if (d < rest)
                consume(d, false);
    }
}

constexpr size_t kStreamMaxLds = 64 * 1024;  // per workgroup (static limit of a launch without opt-in)
constexpr size_t kCuLds = 160 * 1024;
constexpr int kComputeUnits = 256;

// LDS bytes the streaming kernel needs for this problem, 0 if it cannot serve it (more than 8 short strings, a depth
// whose strings do not fit in LDS, binary X strings of an odd number of words)
template <int KIND> size_t stream_lds_bytes(const SkinnyArgs &a)
{
    using T = SkTraits<KIND>;
    constexpr int W = sizeof(typename T::X) == 8 ? 2 : 1;
    if (a.rowsY > 8 || (W == 2 && (a.KW & 1)))
        return 0;
    const int64_t JWn = (a.KW + 64 * W - 1) / (64 * W);
    const int64_t bytes = JWn * 8 * 64 * W * (int64_t)sizeof(typename T::Y) + 8 * 4;
    return bytes <= (int64_t)kStreamMaxLds ? (size_t)bytes : 0;
}

// How the streaming kernel is launched: rows per wave and step, workgroups (of 8 waves) per compute unit, and the
// largest ring depth tried (the depth used is the largest of 8 / 4 / 2 / 1 within it that divides the steps per row).
struct StreamShape {
    int rows_per_wave, wg_per_cu, max_depth;
};

// workgroups of 8 waves in the grid: one per 8 row groups, at most wg_per_cu (and what fits in its LDS) per compute unit
template <int KIND, int R> int stream_grid(const SkinnyArgs &a, size_t lds, int wg_per_cu)
{
    const int groups = (a.rowsX + R - 1) / R;
    const int wgs = (groups + 7) / 8;
    int per_cu = (int)(kCuLds / lds);
    per_cu = per_cu < wg_per_cu ? per_cu : wg_per_cu;
    const int maxwg = kComputeUnits * (per_cu < 1 ? 1 : per_cu);
    return wgs < maxwg ? wgs : maxwg;
}

template <int KIND, int R, bool TR, bool KFULL, int D>
hipError_t launch_stream_inst(const SkinnyArgs &a, size_t lds, int wg_per_cu)
{
    using T = SkTraits<KIND>;
    constexpr int W = sizeof(typename T::X) == 8 ? 2 : 1, WAVES = 8, NS = 8;
    const int JWn = (a.KW + 64 * W - 1) / (64 * W);
    const int groups = (a.rowsX + R - 1) / R;
    const int gx = stream_grid<KIND, R>(a, lds, wg_per_cu);
    hipLaunchKernelGGL((gemm_skinny_stream_kernel<KIND, R, WAVES, TR, NS, KFULL, D>), dim3((unsigned)gx, 1),
                       dim3(64 * WAVES), lds, a.stream, a.Xp, a.Yp, a.rowsX, a.rowsY, a.KW, a.K, a.C, a.ldc, a.c16, JWn,
                       groups);
    return hipGetLastError();
}

template <int KIND, int R, bool TR> hipError_t launch_stream_r(const SkinnyArgs &a, size_t lds, const StreamShape &sh)
{
    using T = SkTraits<KIND>;
    constexpr int W = sizeof(typename T::X) == 8 ? 2 : 1;
    const int JWn = (a.KW + 64 * W - 1) / (64 * W);
    const bool full = a.KW % (64 * W) == 0;
    // ring depth: at most what every working wave has in steps (whole rows of JWn steps, floor(groups / waves) of them
    // or one), at most the shape's limit
    const int groups = (a.rowsX + R - 1) / R;
    const int64_t waves = (int64_t)stream_grid<KIND, R>(a, lds, sh.wg_per_cu) * 8;
    const int64_t min_steps = (int64_t)JWn * (groups / waves > 1 ? groups / waves : 1);
    int d = min_steps >= 8 ? 8 : min_steps >= 4 ? 4 : min_steps >= 2 ? 2 : 1;
    d = d < sh.max_depth ? d : sh.max_depth;
    if constexpr (R == 2)
        d = d < 4 ? d : 4;  // two rows per step: a ring of 8 steps would not leave the registers for 8 waves per SIMD
#define LB_STREAM_D(FULL)                                                                              \
    (d == 8   ? launch_stream_inst<KIND, R, TR, FULL, (R == 2 ? 4 : 8)>(a, lds, sh.wg_per_cu)         \
     : d == 4 ? launch_stream_inst<KIND, R, TR, FULL, 4>(a, lds, sh.wg_per_cu)                         \
     : d == 2 ? launch_stream_inst<KIND, R, TR, FULL, 2>(a, lds, sh.wg_per_cu)                         \
              : launch_stream_inst<KIND, R, TR, FULL, 1>(a, lds, sh.wg_per_cu))
    return full ? LB_STREAM_D(true) : LB_STREAM_D(false);
#undef LB_STREAM_D
}

template <int KIND> hipError_t launch_stream(const SkinnyArgs &a, bool tr, size_t lds, const StreamShape &sh)
{
    if (sh.rows_per_wave == 2)
        return tr ? launch_stream_r<KIND, 2, true>(a, lds, sh) : launch_stream_r<KIND, 2, false>(a, lds, sh);
    return tr ? launch_stream_r<KIND, 1, true>(a, lds, sh) : launch_stream_r<KIND, 1, false>(a, lds, sh);
}

// configurations 8 .. 13 of the benchmark hook force the streaming kernel in these shapes
constexpr StreamShape kStreamForced[] = {{1, 2, 4}, {2, 2, 4}, {1, 4, 4}, {2, 4, 4}, {1, 2, 8}, {1, 4, 8}};
constexpr int kChunkedConfigs = 8;
constexpr int kStreamConfigs = (int)(sizeof(kStreamForced) / sizeof(kStreamForced[0]));

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
    // at most 8 short strings that fit in LDS whole: the streaming kernel (configurations 8 and up force it in a given
    // shape; a problem it cannot serve falls back to the chunked kernel)
    if (cfg < 0 || cfg >= kChunkedConfigs) {
        const size_t lds = stream_lds_bytes<KIND>(a);
        // Measured (cold operand, 4096 .. 131072 rows, depth 4096 .. 32768): the streaming kernel is 0-20 % faster than
        // the chunked one except on the longest ternary-binary streams, which the chunked kernel already runs at the
        // rate of a read-only kernel; two rows per wave pay from 32768 rows on (binary X: from 16384; ternary x ternary:
        // never).
        constexpr bool kTbn = KIND == KIND_TBN || KIND == KIND_TBN_SV;
        const bool chunked_better = cfg < 0 && kTbn && a.rowsX >= 65536 && a.KW >= 256;
        if (lds > 0 && !chunked_better) {
            // ternary x ternary keeps one row per wave at every size (two gain nothing on long streams and lose 8 %
            // at 16384 rows)
            const int two_from = KIND == KIND_BNN ? 16384 : KIND == KIND_TNN ? 0x7fffffff : 32768;
            const StreamShape sh = cfg >= kChunkedConfigs ? kStreamForced[cfg - kChunkedConfigs]
                                                          : StreamShape{a.rowsX >= two_from ? 2 : 1, 4, 4};
            return launch_stream<KIND>(a, tr, lds, sh);
        }
        cfg = -1;
    }
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

int skinny_num_configs() { return kChunkedConfigs + kStreamConfigs; }
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
