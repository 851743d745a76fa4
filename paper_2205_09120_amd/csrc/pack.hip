// Packing kernels: int8 {-1,0,+1} / {-1,+1} matrices -> depth-contiguous 64-bit bit-plane words
// (encodings of Section III-A of the paper; the role of PackNRowsA / PackNColsB in its Algorithms 1 and 2).
//
// Output format: see include/lowbit_gemm.h.  All kernels are HBM-bound streaming kernels: 1 byte read per
// element, 1 or 2 bits written.
//   * depth-contiguous source (stride_k == 1, e.g. A row-major): four lanes share one 64-bit word; each lane
//     reads 16 consecutive bytes (one 128-bit load, fully coalesced), extracts 16 plus and 16 minus bits, and the
//     quad exchanges its pieces with DPP moves so that every lane stores one 32-bit piece of the output.
//   * depth-strided source (stride_r == 1, e.g. B row-major, packed along its columns): a lane reads one dword
//     = 4 adjacent bit strings at one depth position (coalesced along the strings), shifts the sign / non-zero
//     bit of each byte into four per-byte shift registers (8 depth positions per byte), transposes the bytes in
//     registers, and the workgroup writes its 128 strings x 8 words tile through LDS so that stores are
//     contiguous along the depth words.
// Source loads go through memcpy, which the compiler lowers to the same dword / dwordx4 loads for any address:
// global memory needs no alignment for them, so odd leading dimensions and misaligned pointers take the same
// kernels (a leading dimension of 4600 instead of 4608 costs a few percent, not the 9x of byte loads).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

constexpr uint32_t kHi = 0x80808080u, kLo = 0x7f7f7f7fu;

// bit 7 of each byte: byte is negative / byte is positive
__device__ __forceinline__ uint32_t neg7(uint32_t x) { return x & kHi; }
__device__ __forceinline__ uint32_t pos7(uint32_t x) { return ((x & kLo) + kLo) & ~x & kHi; }

// gather bits 7,15,23,31 into bits 0..3
__device__ __forceinline__ uint32_t gather4(uint32_t m)
{
    const uint32_t y = (m >> 7) | (m >> 14);
    return (y | (y >> 14)) & 0xfu;
}

__device__ __forceinline__ uint32_t bits16(const uint4 &v, bool plus)
{
    uint32_t a = plus ? pos7(v.x) : neg7(v.x);
    uint32_t b = plus ? pos7(v.y) : neg7(v.y);
    uint32_t c = plus ? pos7(v.z) : neg7(v.z);
    uint32_t d = plus ? pos7(v.w) : neg7(v.w);
    return gather4(a) | (gather4(b) << 4) | (gather4(c) << 8) | (gather4(d) << 12);
}

// value of `x` held by lane (quad base + Q) of every quad
template <int Q> __device__ __forceinline__ uint32_t quad_bcast(uint32_t x)
{
    constexpr int ctrl = Q | (Q << 2) | (Q << 4) | (Q << 6);  // quad_perm:[Q,Q,Q,Q]
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, ctrl, 0xf, 0xf, true);
}

// ---------------------------------------------------------------------------------------------------------
// depth-contiguous source.  Thread t handles bytes [16*(t%4), +16) of word (t/4) in row-major (r, w) order.
template <bool TERNARY>
__global__ __launch_bounds__(256) void pack_kcontig_kernel(const int8_t *__restrict__ src, int64_t rows, int64_t K,
                                                           int64_t KW, int64_t stride_r, uint32_t *__restrict__ dst)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t word = t >> 2;  // r*KW + w
    const int q = (int)(t & 3);
    const bool live = word < rows * KW;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (live) {
        const int64_t r = word / KW, w = word - r * KW;
        const int64_t k0 = w * 64 + q * 16;
        const int8_t *p = src + r * stride_r + k0;
        if (k0 + 16 <= K) {
            __builtin_memcpy(&v, p, 16);
        } else if (k0 < K && K >= 16) {
            // last piece of a row: fetch the 16 bytes that end at K and shift the ones before k0 out
            uint64_t h[2];
            __builtin_memcpy(h, src + r * stride_r + (K - 16), 16);
            const int sb = 8 * (int)(k0 + 16 - K);  // 8 .. 120 bits
            const uint64_t lo = sb >= 64 ? h[1] >> (sb - 64) : (h[0] >> sb) | (h[1] << (64 - sb));
            const uint64_t hi = sb >= 64 ? 0 : h[1] >> sb;
            v = make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
        } else if (k0 < K) {
            uint32_t tmp[4] = {0u, 0u, 0u, 0u};
            for (int i = 0; i < (int)(K - k0); ++i)
                tmp[i >> 2] |= (uint32_t)(uint8_t)p[i] << (8 * (i & 3));
            v = make_uint4(tmp[0], tmp[1], tmp[2], tmp[3]);
        }
    }
    const uint32_t mine = bits16(v, false) | (TERNARY ? (bits16(v, true) << 16) : 0u);  // minus low, plus high
    const uint32_t p0 = quad_bcast<0>(mine), p1 = quad_bcast<1>(mine), p2 = quad_bcast<2>(mine),
                   p3 = quad_bcast<3>(mine);
    if (!live)
        return;
    if (TERNARY) {
        // dwords of the 16-byte entry: plus_lo, plus_hi, minus_lo, minus_hi
        uint32_t out;
        if (q == 0)
            out = (p0 >> 16) | (p1 & 0xffff0000u);
        else if (q == 1)
            out = (p2 >> 16) | (p3 & 0xffff0000u);
        else if (q == 2)
            out = (p0 & 0xffffu) | (p1 << 16);
        else
            out = (p2 & 0xffffu) | (p3 << 16);
        dst[word * 4 + q] = out;
    } else {
        if (q == 0)
            dst[word * 2] = (p0 & 0xffffu) | (p1 << 16);
        else if (q == 1)
            dst[word * 2 + 1] = (p2 & 0xffffu) | (p3 << 16);
    }
}

// ---------------------------------------------------------------------------------------------------------
// depth-strided source.  Workgroup tile: 128 bit strings x 8 depth words.  Thread (quad = tid%32, w = tid/32).
template <bool TERNARY>
__global__ __launch_bounds__(256) void pack_kstrided_kernel(const int8_t *__restrict__ src, int64_t rows, int64_t K,
                                                            int64_t KW, int64_t stride_k, uint32_t *__restrict__ dst,
                                                            int64_t nRB)
{
    constexpr int ED = TERNARY ? 4 : 2;       // dwords per output entry
    // LDS tile: 128 strings x 8 entries (one entry = one depth word of a string: 16 bytes ternary, 8 bytes binary).
    // The LDS moves 128 bytes per clock, i.e. the entries of 8 (ternary) or 16 (binary) consecutive lanes, which must
    // fall into different 16- / 8-byte columns of that window.  String quad*4 + i sits in row i*32 + quad and entry e
    // of row r in slot e ^ ((r >> SW) & 7): the lanes of one write hold consecutive rows and the same e, the lanes of
    // one read all 8 entries of one row (ternary) or of two rows that differ in bit 0 (binary).  Measured: bank-conflict
    // cycles fell from 47 % of the LDS-active cycles (padded tile) to 25 %, binary packing is 10 % faster.
    using Entry = typename std::conditional<TERNARY, uint4, uint2>::type;
    constexpr int SW = TERNARY ? 0 : 1;
    __shared__ Entry tile[128 * 8];
    const int64_t rb = blockIdx.x % nRB, wb = blockIdx.x / nRB;
    const int quad = threadIdx.x & 31, wl = threadIdx.x >> 5;
    const int64_t r0 = rb * 128 + quad * 4;
    const int64_t w = wb * 8 + wl;
    const int64_t kbase = w * 64;

    uint32_t neg[8], pos[8];
    // Workgroups whose 128 strings x 512 depth positions lie inside the matrix take straight-line loads (a load
    // inside a divergent branch forces a wait right behind it); edge workgroups take the guarded path.
    const bool interior = (rb + 1) * 128 <= rows && (wb + 1) * 512 <= K;
    if (interior) {
        const int8_t *p = src + kbase * stride_k + r0;
#pragma unroll
        for (int kb = 0; kb < 8; ++kb) {
            uint32_t x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                __builtin_memcpy(&x[j], p, 4);
                p += stride_k;
            }
            uint32_t an = 0u, ap = 0u;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                an = (an >> 1) | neg7(x[j]);
                if (TERNARY)
                    ap = (ap >> 1) | pos7(x[j]);
            }
            neg[kb] = an;
            pos[kb] = ap;
        }
    } else {
#pragma unroll
        for (int kb = 0; kb < 8; ++kb) {
            uint32_t an = 0u, ap = 0u;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int64_t k = kbase + kb * 8 + j;
                uint32_t x = 0u;
                if (k < K && r0 < rows) {
                    const int8_t *p = src + k * stride_k + r0;
                    if (r0 + 4 <= rows) {
                        __builtin_memcpy(&x, p, 4);
                    } else {
                        for (int i = 0; i < (int)(rows - r0); ++i)
                            x |= (uint32_t)(uint8_t)p[i] << (8 * i);
                    }
                }
                an = (an >> 1) | neg7(x);
                if (TERNARY)
                    ap = (ap >> 1) | pos7(x);
            }
            neg[kb] = an;  // byte i = 8 depth bits of string r0+i
            pos[kb] = ap;
        }
    }
    // byte transpose: string i gets bytes i of neg[0..3] (low dword) and of neg[4..7] (high dword)
    auto transpose4 = [](const uint32_t *a, uint32_t *o) __attribute__((always_inline)) {
        const uint32_t t0 = __builtin_amdgcn_perm(a[1], a[0], 0x05010400u), t1 = __builtin_amdgcn_perm(a[1], a[0], 0x07030602u);
        const uint32_t t2 = __builtin_amdgcn_perm(a[3], a[2], 0x05010400u), t3 = __builtin_amdgcn_perm(a[3], a[2], 0x07030602u);
        o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
        o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
        o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
        o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
    };
    uint32_t nlo[4], nhi[4], plo[4], phi[4];
    transpose4(neg, nlo);
    transpose4(neg + 4, nhi);
    if (TERNARY) {
        transpose4(pos, plo);
        transpose4(pos + 4, phi);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = i * 32 + quad;
        Entry e;
        if constexpr (TERNARY)
            e = make_uint4(plo[i], phi[i], nlo[i], nhi[i]);
        else
            e = make_uint2(nlo[i], nhi[i]);
        tile[row * 8 + (wl ^ ((row >> SW) & 7))] = e;
    }
    __syncthreads();
    // write out: the 8 entries of a string are contiguous in dst; a thread moves one entry per round
    constexpr int G = TERNARY ? 1 : 2;  // strings whose entries one LDS clock moves
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int idx = it * 256 + threadIdx.x;
        const int e = idx & 7, t = idx >> 3;
        const int rl = (t % G) * 4 + ((t / G) % 4) + (t / (4 * G)) * (4 * G);  // string within the tile
        const int row = (rl & 3) * 32 + (rl >> 2);
        const Entry v = tile[row * 8 + (e ^ ((row >> SW) & 7))];
        const int64_t r = rb * 128 + rl;
        const int64_t ww = wb * 8 + e;
        if (r < rows && ww < KW)
            *reinterpret_cast<Entry *>(dst + (r * KW + ww) * ED) = v;
    }
}

}  // namespace

hipError_t launch_pack(bool ternary, const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k,
                       uint64_t *dst, hipStream_t stream)
{
    const int64_t KW = (K + 63) / 64;
    const int64_t words = rows * KW;
    if (words == 0)
        return hipSuccess;
    uint32_t *d32 = reinterpret_cast<uint32_t *>(dst);
    // the C ABI admits exactly two layouts: depth-contiguous (stride_k == 1) and depth-strided (stride_r == 1)
    if (stride_k == 1) {
        const int64_t blocks = (words * 4 + 255) / 256;
        if (blocks > 0x7fffffffLL)
            return hipErrorInvalidConfiguration;
        if (ternary)
            hipLaunchKernelGGL(pack_kcontig_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, src, rows, K,
                               KW, stride_r, d32);
        else
            hipLaunchKernelGGL(pack_kcontig_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, src, rows, K,
                               KW, stride_r, d32);
    } else if (stride_r == 1) {
        const int64_t nRB = (rows + 127) / 128, nWB = (KW + 7) / 8;
        const int64_t blocks = nRB * nWB;
        if (blocks > 0x7fffffffLL)
            return hipErrorInvalidConfiguration;
        if (ternary)
            hipLaunchKernelGGL(pack_kstrided_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, src, rows, K,
                               KW, stride_k, d32, nRB);
        else
            hipLaunchKernelGGL(pack_kstrided_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, src, rows, K,
                               KW, stride_k, d32, nRB);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace lowbit
