// 4-bit unsigned quantized GEMM with zero points on the matrix cores: the stand-in for the paper's U4 comparison
// algorithm (Table II, Section IV; the quantized product and its zero-point expansion are eq. (2) and (3)).
//
// gfx950 has no 4-bit integer matrix instruction, but its scaled MFMA takes 6-bit floats (1 sign, 2 exponent, 3 mantissa
// bits, bias 1) at a higher rate than 8-bit operands (published: twice; measured here: 1.6 times), and with a block scale of 2 that type represents every integer 0..15 exactly
// (0, 0.5, ..., 7.5 doubled).  Products of such values and their fp32 sums are exact while the sum stays below 2^24,
// i.e. for K <= 74565 (15 * 15 * K < 2^24): the result is the integer product, bit for bit.
//
// Operand format ("fragment-major", written by pack_u4): rows padded to multiples of 32, depth to multiples of 128.
// One fragment = 32 rows x 64 depth positions = the operand of one v_mfma_scale_f32_32x32x64_f8f6f4: lane 32*h + i of
// the wavefront holds depth positions 32*h .. 32*h+31 of row i as 192 bits (position j in bits 6j .. 6j+5).  A fragment
// is stored as three planes of 64 lanes x 8 bytes (plane p = bits 64p .. 64p+63 of every lane), 1536 bytes, so a wave
// reads it with three conflict-free ds_read_b64; fragments are ordered by row block, then depth block.  Global memory
// therefore goes to LDS as a plain contiguous copy (global_load_lds_dwordx4), with no transposes or swizzles: like the
// paper's reordered Ablock / Bblock buffers (Section III), the packing step writes exactly what the multiply reads.
//
// The same kernel also multiplies ternary / binary operands ({-1, 0, +1}: the paper's own value sets, Section III-A)
// stored as 4-bit floats (1 sign, 2 exponent, 1 mantissa bit, bias 1: 0 and +-1 are exact), 16 bytes per lane and
// fragment, on the same instruction at its 4-bit rate: what the matrix cores of this chip do with the operands that
// the paper multiplies with AND / XOR / popcount (pack_t4, gemm_t4_mfma).
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <type_traits>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kFragBytes = 1536;          // 32 rows x 64 depth positions x 6 bits
constexpr int kSegBytes = 2 * kFragBytes; // one row block x 128 depth positions: the unit a depth stage moves
constexpr int kScaleTwo = (int)0x80808080u;  // block scale 2^(128 - 127) in every byte, whichever the opsel picks
constexpr int kScaleOne = (int)0x7f7f7f7fu;  // block scale 1
constexpr int kComputeUnits = 256;           // MI355X
constexpr int kFrag4Bytes = 1024;            // 4-bit floats: 32 rows x 64 depth positions x 4 bits

std::atomic<int> g_u4_forced{-1};  // benchmark hook; read once per call

// -------------------------------------------------------------------------------------------------- packing

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t *p, int64_t n, int32_t v)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n)
        p[i] = v;
}

// Four values 0..15 in the bytes of x -> their four 6-bit codes in the bytes of the result.
// code(v) = 4v for v < 4, 2v + 8 for 4 <= v < 8, v + 16 from 8 on  =  4v - max(0, 2v - 8) - max(0, v - 8),
// evaluated on all four bytes at once (no byte ever borrows from its neighbour).
__device__ __forceinline__ uint32_t codes4(uint32_t x)
{
    const uint32_t ge8 = (x >> 3) & 0x01010101u;
    const uint32_t ge4 = ((x >> 2) | (x >> 3)) & 0x01010101u;
    const uint32_t t1 = x & (ge8 * 7u);                            // max(0, v - 8)
    const uint32_t t2 = ((x - (ge4 << 2)) << 1) & (ge4 * 0xffu);   // max(0, 2v - 8)
    return (x << 2) - t2 - t1;
}

// The four 6-bit codes in the bytes of c, packed into 24 bits.
__device__ __forceinline__ uint64_t squeeze4(uint32_t c)
{
    return (uint64_t)((c & 0x3fu) | ((c >> 2) & 0xfc0u) | ((c >> 4) & 0x3f000u) | ((c >> 6) & 0xfc0000u));
}

// 32 values (four per dword, low nibbles) -> the 192-bit string of their codes; their sum is added to `sum`.
__device__ __forceinline__ void encode32(const uint32_t (&w)[8], uint64_t &q0, uint64_t &q1, uint64_t &q2, uint32_t &sum)
{
    uint64_t f[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const uint32_t x = w[t] & 0x0f0f0f0fu;
        sum = __builtin_amdgcn_sad_u8(x, 0u, sum);
        f[t] = squeeze4(codes4(x));
    }
    q0 = f[0] | (f[1] << 24) | (f[2] << 48);
    q1 = (f[2] >> 16) | (f[3] << 8) | (f[4] << 32) | (f[5] << 56);
    q2 = (f[5] >> 8) | (f[6] << 16) | (f[7] << 40);
}

// Thread (i = tid % 32, gg = tid / 32) of block (rb, chunk) encodes 32 consecutive depth positions (group g) of row
// 32*rb + i per iteration, groups g = 8*u + gg for the units u = chunk, chunk + gridDim.y, ...: the 32 threads of
// one gg write 256 contiguous bytes of a plane, and the eight groups of a unit cover two cache lines of every row.
// Depth-contiguous source: element (r, k) at src[r*stride + k].  Only the low four bits of a source byte count.  The
// row sums are added into sums[] (cleared beforehand) with one atomic per row and block.
__global__ __launch_bounds__(256) void pack_u4_kernel(const uint8_t *__restrict__ src, int64_t rows, int64_t K,
                                                      int64_t stride, uint8_t *__restrict__ dst,
                                                      int32_t *__restrict__ sums, int KB)
{
    __shared__ int red[256];
    const int tid = threadIdx.x, i = tid & 31, gg = tid >> 5;
    const int64_t rb = blockIdx.x, r = rb * 32 + i;
    const int G = KB * 2, units = (G + 7) / 8;
    const bool row_ok = r < rows;
    uint32_t psum = 0;
    for (int u = blockIdx.y; u < units; u += gridDim.y) {
        const int g = u * 8 + gg;
        if (g >= G)
            continue;
        const int64_t k0 = (int64_t)g * 32;
        uint32_t w[8];
#pragma unroll
        for (int t = 0; t < 8; ++t)
            w[t] = 0u;
        if (row_ok && k0 < K) {
            if (k0 + 32 <= K) {
                uint4 lo, hi;
                const uint8_t *p = src + r * stride + k0;
                __builtin_memcpy(&lo, p, 16);
                __builtin_memcpy(&hi, p + 16, 16);
                w[0] = lo.x; w[1] = lo.y; w[2] = lo.z; w[3] = lo.w;
                w[4] = hi.x; w[5] = hi.y; w[6] = hi.z; w[7] = hi.w;
            } else {
#pragma unroll
                for (int j = 0; j < 32; ++j) {
                    const int64_t k = k0 + j;
                    uint32_t v = 0u;
                    if (k < K)
                        v = src[r * stride + k];
                    w[j >> 2] |= v << (8 * (j & 3));
                }
            }
        }
        uint64_t q0, q1, q2;
        encode32(w, q0, q1, q2, psum);
        uint8_t *o = dst + (rb * KB + (g >> 1)) * (int64_t)kFragBytes + ((g & 1) * 32 + i) * 8;
        *reinterpret_cast<uint64_t *>(o) = q0;
        *reinterpret_cast<uint64_t *>(o + 512) = q1;
        *reinterpret_cast<uint64_t *>(o + 1024) = q2;
    }
    red[tid] = (int)psum;
    __syncthreads();
    if (gg == 0 && row_ok) {
        int s = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t)
            s += red[t * 32 + i];
        atomicAdd(&sums[r], s);
    }
}

// Depth-strided source (element (r, k) at src[k*stride + r], the K x rows layout of a right operand): a block covers
// 128 rows; lane (q = lane % 32, hh = lane / 32) of wave w loads, for each of the 32 depth positions of group
// g = 8*u + 2*w + hh, the four bytes of rows 4q .. 4q+3 -- 32 lanes read one whole 128-byte line of a depth row --,
// transposes the 4 x 32 bytes in registers (4 x 4 byte transposes, v_perm_b32) and encodes its four rows.  Their four
// 8-byte pieces of a plane are adjacent slots: 32-byte stores, 256 contiguous bytes per eight lanes.
__global__ __launch_bounds__(256) void pack_u4_strided_kernel(const uint8_t *__restrict__ src, int64_t rows, int64_t K,
                                                              int64_t stride, uint8_t *__restrict__ dst,
                                                              int32_t *__restrict__ sums, int KB, int64_t RB)
{
    __shared__ int red[4][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, q = lane & 31, hh = lane >> 5;
    const int64_t r0 = (int64_t)blockIdx.x * 128 + 4 * q;
    const int64_t rb = r0 >> 5;
    const int G = KB * 2, units = (G + 7) / 8;
    const bool quad_ok = r0 + 3 < rows;
    uint32_t psum[4] = {0u, 0u, 0u, 0u};
    for (int u = blockIdx.y; u < units; u += gridDim.y) {
        const int g = u * 8 + wave * 2 + hh;
        if (g >= G || rb >= RB)
            continue;
        const int64_t k0 = (int64_t)g * 32;
        uint32_t w[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int64_t k = k0 + j;
            uint32_t v = 0u;
            if (k < K) {
                const uint8_t *p = src + k * stride + r0;
                if (quad_ok) {
                    __builtin_memcpy(&v, p, 4);
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (r0 + b < rows)
                            v |= (uint32_t)p[b] << (8 * b);
                }
            }
            w[j] = v;
        }
        uint64_t out[3][4];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            uint32_t x[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                // byte rr of w[4t .. 4t+3]: two rounds of byte interleaving
                const uint32_t a = __builtin_amdgcn_perm(w[4 * t + 1], w[4 * t], rr < 2 ? 0x05010400u : 0x07030602u);
                const uint32_t b = __builtin_amdgcn_perm(w[4 * t + 3], w[4 * t + 2], rr < 2 ? 0x05010400u : 0x07030602u);
                x[t] = __builtin_amdgcn_perm(b, a, (rr & 1) ? 0x07060302u : 0x05040100u);
            }
            encode32(x, out[0][rr], out[1][rr], out[2][rr], psum[rr]);
        }
        uint8_t *o = dst + (rb * KB + (g >> 1)) * (int64_t)kFragBytes + ((g & 1) * 32 + 4 * (q & 7)) * 8;
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            *reinterpret_cast<ulonglong2 *>(o + p * 512) = make_ulonglong2(out[p][0], out[p][1]);
            *reinterpret_cast<ulonglong2 *>(o + p * 512 + 16) = make_ulonglong2(out[p][2], out[p][3]);
        }
    }
#pragma unroll
    for (int rr = 0; rr < 4; ++rr)
        red[rr][tid] = (int)psum[rr];
    __syncthreads();
    if (tid < 32) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            int s = 0;
#pragma unroll
            for (int t = 0; t < 8; ++t)
                s += red[rr][t * 32 + q];
            if (r0 + rr < rows)
                atomicAdd(&sums[r0 + rr], s);
        }
    }
}

// ---- ternary / binary values as 4-bit floats

// Four int8 values in the bytes of x, taken by sign -> their four 4-bit codes (+1: 0b0010, -1: 0b1010, 0: 0) in 16 bits.
__device__ __forceinline__ uint32_t codes4_fp4(uint32_t x)
{
    const uint32_t neg = x & 0x80808080u;
    const uint32_t nz = (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;  // 0x80 in every nonzero byte
    const uint32_t c = (nz >> 6) | (neg >> 4);                                  // one code per byte (low nibble)
    return (c & 0xfu) | ((c >> 4) & 0xf0u) | ((c >> 8) & 0xf00u) | ((c >> 12) & 0xf000u);
}

__device__ __forceinline__ uint4 encode32_fp4(const uint32_t (&w)[8])
{
    uint32_t f[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
        f[t] = codes4_fp4(w[t]);
    return make_uint4(f[0] | (f[1] << 16), f[2] | (f[3] << 16), f[4] | (f[5] << 16), f[6] | (f[7] << 16));
}

// Same thread mapping as pack_u4_kernel; a thread writes the 16 bytes of its slot.
__global__ __launch_bounds__(256) void pack_t4_kernel(const int8_t *__restrict__ src, int64_t rows, int64_t K,
                                                      int64_t stride, uint8_t *__restrict__ dst, int KB)
{
    const int tid = threadIdx.x, i = tid & 31, gg = tid >> 5;
    const int64_t rb = blockIdx.x, r = rb * 32 + i;
    const int G = KB * 2, units = (G + 7) / 8;
    const bool row_ok = r < rows;
    for (int u = blockIdx.y; u < units; u += gridDim.y) {
        const int g = u * 8 + gg;
        if (g >= G)
            continue;
        const int64_t k0 = (int64_t)g * 32;
        uint32_t w[8];
#pragma unroll
        for (int t = 0; t < 8; ++t)
            w[t] = 0u;
        if (row_ok && k0 < K) {
            if (k0 + 32 <= K) {
                uint4 lo, hi;
                const int8_t *p = src + r * stride + k0;
                __builtin_memcpy(&lo, p, 16);
                __builtin_memcpy(&hi, p + 16, 16);
                w[0] = lo.x; w[1] = lo.y; w[2] = lo.z; w[3] = lo.w;
                w[4] = hi.x; w[5] = hi.y; w[6] = hi.z; w[7] = hi.w;
            } else {
#pragma unroll
                for (int j = 0; j < 32; ++j) {
                    const int64_t k = k0 + j;
                    uint32_t v = 0u;
                    if (k < K)
                        v = (uint8_t)src[r * stride + k];
                    w[j >> 2] |= v << (8 * (j & 3));
                }
            }
        }
        uint8_t *o = dst + (rb * KB + (g >> 1)) * (int64_t)kFrag4Bytes + ((g & 1) * 32 + i) * 16;
        *reinterpret_cast<uint4 *>(o) = encode32_fp4(w);
    }
}

// Same thread mapping as pack_u4_strided_kernel; the four rows of a lane are four adjacent 16-byte slots.
__global__ __launch_bounds__(256) void pack_t4_strided_kernel(const int8_t *__restrict__ src, int64_t rows, int64_t K,
                                                              int64_t stride, uint8_t *__restrict__ dst, int KB,
                                                              int64_t RB)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, q = lane & 31, hh = lane >> 5;
    const int64_t r0 = (int64_t)blockIdx.x * 128 + 4 * q;
    const int64_t rb = r0 >> 5;
    const int G = KB * 2, units = (G + 7) / 8;
    const bool quad_ok = r0 + 3 < rows;
    for (int u = blockIdx.y; u < units; u += gridDim.y) {
        const int g = u * 8 + wave * 2 + hh;
        if (g >= G || rb >= RB)
            continue;
        const int64_t k0 = (int64_t)g * 32;
        uint32_t w[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int64_t k = k0 + j;
            uint32_t v = 0u;
            if (k < K) {
                const int8_t *p = src + k * stride + r0;
                if (quad_ok) {
                    __builtin_memcpy(&v, p, 4);
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (r0 + b < rows)
                            v |= (uint32_t)(uint8_t)p[b] << (8 * b);
                }
            }
            w[j] = v;
        }
        uint8_t *o = dst + (rb * KB + (g >> 1)) * (int64_t)kFrag4Bytes + ((g & 1) * 32 + 4 * (q & 7)) * 16;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            uint32_t x[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const uint32_t a = __builtin_amdgcn_perm(w[4 * t + 1], w[4 * t], rr < 2 ? 0x05010400u : 0x07030602u);
                const uint32_t b = __builtin_amdgcn_perm(w[4 * t + 3], w[4 * t + 2], rr < 2 ? 0x05010400u : 0x07030602u);
                x[t] = __builtin_amdgcn_perm(b, a, (rr & 1) ? 0x07060302u : 0x05040100u);
            }
            *reinterpret_cast<uint4 *>(o + rr * 16) = encode32_fp4(x);
        }
    }
}

// -------------------------------------------------------------------------------------------------- product

// WM x WN waves, each RM x RN MFMA blocks of 32 x 32: workgroup tile (32*RM*WM) x (32*RN*WN).  Every wave both issues
// its share of the direct-to-LDS loads (they occupy no registers) STAGES - 1 depth stages of 128 positions ahead and
// multiplies.  One barrier per stage: before it a wave waits for its own loads of the stage about to be read; behind it
// every wave has finished reading the stage before, whose buffer the loads issued next overwrite.
// Row blocks beyond the operand (ragged M, N) re-read the operand's last row block: always in bounds, and the
// products they feed are never stored.
// FMT is the element format of both operands as the instruction numbers them: 2 = 6-bit floats (24 bytes per lane and
// fragment, three planes of 8, block scale 2, zero-point epilogue), 4 = 4-bit floats (16 bytes per lane, scale 1, no
// zero points: sumA / sumB are not read).
template <int FMT, int WM, int WN, int RM, int RN, int STAGES>
__global__ __launch_bounds__(64 * WM * WN) void gemm_mx_kernel(
    const uint8_t *__restrict__ Ap, const uint8_t *__restrict__ Bp, const int32_t *__restrict__ sumA,
    const int32_t *__restrict__ sumB, int M, int N, int K, int KB2, int RBA, int RBB, int32_t *__restrict__ C,
    int64_t ldc, int nMB, int nNB, int tiles_per_xcd, int zA, int zB)
{
    static_assert(FMT == 2 || FMT == 4, "6-bit or 4-bit floats");
    constexpr int kFragBytes = FMT == 2 ? 1536 : kFrag4Bytes;  // shadows the 6-bit constant of the packing kernels
    constexpr int kSegBytes = 2 * kFragBytes;                  // one row block x 128 depth positions
    constexpr int LPS = kSegBytes / 1024;                      // wave-wide 1 KB loads per segment
    constexpr int kScale = FMT == 2 ? kScaleTwo : kScaleOne;
    constexpr int NW = WM * WN;
    constexpr int SA = RM * WM, SB = RN * WN;          // row-block segments of A and of B per stage
    constexpr int STAGE = (SA + SB) * kSegBytes;
    constexpr int LOADS = (SA + SB) * LPS;             // wave-wide 1 KB loads per stage
    constexpr int LW = LOADS / NW;                     // ... per wave
    static_assert(LOADS % NW == 0 && (STAGES - 2) * LW < 64 && STAGES >= 2, "load split / vmcnt is a 6-bit counter");
    static_assert(STAGES * STAGE <= 160 * 1024, "LDS");

    __shared__ __attribute__((aligned(1024))) uint8_t smem[STAGES * STAGE];

    const int bid = blockIdx.x;
    const int idx = (bid & 7) * tiles_per_xcd + (bid >> 3);   // consecutive tiles stay on one XCD (one L2)
    if ((bid >> 3) >= tiles_per_xcd || idx >= nMB * nNB)
        return;
    const int nb = idx / nMB, mb = idx - nb * nMB;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wm = wave % WM, wn = wave / WM;

    const uint8_t *src[LW];
#pragma unroll
    for (int t = 0; t < LW; ++t) {
        const int q = wave * LW + t, seg = q / LPS, part = q - seg * LPS;
        const uint8_t *base;
        if (seg < SA) {
            int rb = mb * SA + seg;
            rb = rb < RBA ? rb : RBA - 1;
            base = Ap + (int64_t)rb * KB2 * kSegBytes;
        } else {
            int cb = nb * SB + (seg - SA);
            cb = cb < RBB ? cb : RBB - 1;
            base = Bp + (int64_t)cb * KB2 * kSegBytes;
        }
        src[t] = base + part * 1024 + lane * 16;
    }
    // The direct-to-LDS loads are inline assembly: the compiler would otherwise order every LDS read behind ALL
    // outstanding direct loads (vmcnt(0)), which serialises the ring of stages.  Written this way it does not know
    // that these loads write LDS; what orders them against the fragment reads is the stage barrier, which follows each
    // wave's own explicit vmcnt wait.  M0 carries the LDS address of a wave-wide load (lane l lands at M0 + 16*l).
    auto issue_one = [&](int s, int t) __attribute__((always_inline)) {
        const uint32_t st = (uint32_t)(uintptr_t)smem + (uint32_t)((s % STAGES) * STAGE + (wave * LW + t) * 1024);
        const uint8_t *g = src[t] + (int64_t)s * kSegBytes;
        // one wait state between the write of M0 and the load that reads it (the compiler inserts it for its own
        // direct loads; it does not look into assembly statements)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(st), "v"(g) : "memory", "m0");
    };
    auto issue = [&](int s) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < LW; ++t)
            issue_one(s, t);
    };

    v16f acc[RM][RN];
#pragma unroll
    for (int i = 0; i < RM; ++i)
#pragma unroll
        for (int j = 0; j < RN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.f;

    // Fragments of the next depth step are read while the MFMAs of the current one run (two fragment sets alternate).
    const int a_off = (wm * RM) * kSegBytes + lane * (FMT == 2 ? 8 : 16);
    const int b_off = (SA + wn * RN) * kSegBytes + lane * (FMT == 2 ? 8 : 16);
    auto frag = [&](const uint8_t *p) __attribute__((always_inline)) {
        if constexpr (FMT == 2) {
            const uint2 q0 = *reinterpret_cast<const uint2 *>(p);
            const uint2 q1 = *reinterpret_cast<const uint2 *>(p + 512);
            const uint2 q2 = *reinterpret_cast<const uint2 *>(p + 1024);
            return v8i{(int)q0.x, (int)q0.y, (int)q1.x, (int)q1.y, (int)q2.x, (int)q2.y, 0, 0};
        } else {
            const uint4 q = *reinterpret_cast<const uint4 *>(p);
            return v8i{(int)q.x, (int)q.y, (int)q.z, (int)q.w, 0, 0, 0, 0};
        }
    };
    auto read_frags = [&](int s, int ks, v8i(&a)[RM], v8i(&b)[RN]) __attribute__((always_inline)) {
        const uint8_t *st = smem + (s % STAGES) * STAGE + ks * kFragBytes;
#pragma unroll
        for (int i = 0; i < RM; ++i)
            a[i] = frag(st + a_off + i * kSegBytes);
#pragma unroll
        for (int j = 0; j < RN; ++j)
            b[j] = frag(st + b_off + j * kSegBytes);
    };
    auto mfma_rows = [&](v8i(&a)[RM], v8i(&b)[RN], int i0, int i1) __attribute__((always_inline)) {
#pragma unroll
        for (int i = i0; i < i1; ++i)
#pragma unroll
            for (int j = 0; j < RN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], acc[i][j], FMT, FMT, 0, kScale, 0,
                                                                             kScale);
    };
    // "stage s holds its data and the stage before it is free": own loads landed (all but `in_flight` newer ones),
    // then the workgroup barrier
    auto stage_barrier = [&](auto in_flight) __attribute__((always_inline)) {
        constexpr int vm = decltype(in_flight)::value;
        static_assert(vm < 64, "vmcnt is a 6-bit counter");
        __builtin_amdgcn_s_waitcnt((vm & 15) | ((vm >> 4) << 14) | 0x0f70);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    using steady = std::integral_constant<int, (STAGES - 2) * LW>;
    using drain = std::integral_constant<int, 0>;

    // One stage = two depth steps.  What happens at the switch to stage s + 1 depends on how many stages are left
    // (stages up to s + STAGES - 1 have been issued by then): MODE 0 barrier with STAGES - 2 stages in flight, then
    // issue stage s + STAGES; 1 the same barrier, nothing left to issue; 2 barrier with everything landed; 3 last
    // stage, no switch.  Each mode is straight-line code, so that the order written here is the order executed.
    const int nst = KB2;
    v8i fa[2][RM], fb[2][RN];
    for (int s = 0; s < STAGES - 1 && s < nst; ++s)
        issue(s);
    if (STAGES - 1 < nst) {
        stage_barrier(steady{});
        issue(STAGES - 1);
    } else {
        stage_barrier(drain{});
    }
    read_frags(0, 0, fa[0], fb[0]);
    // Per depth step: the first row of MFMAs (the compiler's wait in front of it covers the fragment reads in
    // flight), the reads of the next step -- behind the stage barrier when the step is the last of its stage --, the
    // other rows.
    auto stage_body = [&](auto mode, int s) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode)::value;
        mfma_rows(fa[0], fb[0], 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(s, 1, fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
        mfma_rows(fa[0], fb[0], 1, RM);
        __builtin_amdgcn_sched_barrier(0);
        mfma_rows(fa[1], fb[1], 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (MODE == 0 || MODE == 1) {
            stage_barrier(steady{});
        } else if constexpr (MODE == 2) {
            stage_barrier(drain{});
        }
        if constexpr (MODE != 3)
            read_frags(s + 1, 0, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (MODE == 0 && RM > 1) {
            // the direct loads of stage s + STAGES go out between the remaining MFMAs, not in one burst: a wave
            // that is busy issuing loads issues no MFMAs
            constexpr int SLOTS = RM > 1 ? (RM - 1) * RN : 1, PER = (LW + SLOTS - 1) / SLOTS;
#pragma unroll
            for (int i = 1; i < RM; ++i)
#pragma unroll
                for (int j = 0; j < RN; ++j) {
#pragma unroll
                    for (int c = 0; c < PER; ++c) {
                        const int t = ((i - 1) * RN + j) * PER + c;
                        if (t < LW)
                            issue_one(s + STAGES, t);
                    }
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[1][i], fb[1][j], acc[i][j], FMT, FMT, 0,
                                                                                 kScale, 0, kScale);
                    __builtin_amdgcn_sched_barrier(0);
                }
        } else {
            if constexpr (MODE == 0)
                issue(s + STAGES);
            mfma_rows(fa[1], fb[1], 1, RM);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    {
        int s = 0;
        for (; s + STAGES < nst; ++s)
            stage_body(std::integral_constant<int, 0>{}, s);
        if (s + STAGES == nst) {
            stage_body(std::integral_constant<int, 1>{}, s);
            ++s;
        }
        for (; s + 1 < nst; ++s)
            stage_body(std::integral_constant<int, 2>{}, s);
        stage_body(std::integral_constant<int, 3>{}, s);
    }

    // eq. (3): sum (a - zA)(b - zB) = sum a b - zB * rowsum(A) - zA * colsum(B) + K zA zB.
    // The row sums of all the rows a lane stores to are fetched up front, from indices clamped into range, so that
    // the loads go out together instead of one in front of every guarded store.
    const int m0 = mb * 32 * SA, n0 = nb * 32 * SB;
    if constexpr (FMT == 4) {
#pragma unroll
        for (int j = 0; j < RN; ++j) {
            const int col = n0 + (wn * RN + j) * 32 + (lane & 31);
#pragma unroll
            for (int i = 0; i < RM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + (wm * RM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (col < N && row < M)
                        C[(int64_t)row * ldc + col] = (int)acc[i][j][r];
                }
        }
        return;
    }
    const int kzz = K * zA * zB;
    int rcorr[RM][16];
#pragma unroll
    for (int i = 0; i < RM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + (wm * RM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            rcorr[i][r] = zB * sumA[row < M ? row : M - 1];
        }
#pragma unroll
    for (int j = 0; j < RN; ++j) {
        const int col = n0 + (wn * RN + j) * 32 + (lane & 31);
        const bool col_ok = col < N;
        const int ccorr = kzz - zA * sumB[col_ok ? col : N - 1];
#pragma unroll
        for (int i = 0; i < RM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * RM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (col_ok && row < M)
                    C[(int64_t)row * ldc + col] = (int)acc[i][j][r] + ccorr - rcorr[i][r];
            }
    }
}

template <int FMT, int WM, int WN, int RM, int RN, int STAGES>
hipError_t launch_u4(int64_t M, int64_t N, int64_t K, const uint8_t *Ap, const int32_t *sumA, const uint8_t *Bp,
                     const int32_t *sumB, int zA, int zB, int32_t *C, int64_t ldc, hipStream_t stream)
{
    constexpr int BM = 32 * RM * WM, BN = 32 * RN * WN;
    const int64_t nMB = (M + BM - 1) / BM, nNB = (N + BN - 1) / BN;
    const int64_t tiles = nMB * nNB;
    const int64_t tiles_per_xcd = (tiles + 7) / 8;
    if (tiles_per_xcd * 8 > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((gemm_mx_kernel<FMT, WM, WN, RM, RN, STAGES>), dim3((unsigned)(tiles_per_xcd * 8)),
                       dim3(64 * WM * WN), 0, stream, Ap, Bp, sumA, sumB, (int)M, (int)N, (int)K,
                       (int)((K + 127) / 128), (int)((M + 31) / 32), (int)((N + 31) / 32), C, ldc, (int)nMB, (int)nNB,
                       (int)tiles_per_xcd, zA, zB);
    return hipGetLastError();
}

// Instances: 0 = 256 x 256 tile (4 waves of 128 x 128), 1 = 256 x 256 (8 waves of 64 x 128), 2 = 128 x 128 (4 waves of
// 64 x 64), 3 = 64 x 64 (4 waves of 32 x 32).  Ring depth: 3, 3, 3, 4 stages for 6-bit floats, 4 for 4-bit floats.
template <int FMT>
hipError_t launch_mx_instance(int inst, int64_t M, int64_t N, int64_t K, const uint8_t *Ap, const int32_t *sumA,
                              const uint8_t *Bp, const int32_t *sumB, int zA, int zB, int32_t *C, int64_t ldc,
                              hipStream_t stream)
{
    constexpr int S = FMT == 2 ? 3 : 4;
    switch (inst) {
    case 0: return launch_u4<FMT, 2, 2, 4, 4, S>(M, N, K, Ap, sumA, Bp, sumB, zA, zB, C, ldc, stream);
    case 1: return launch_u4<FMT, 4, 2, 2, 4, S>(M, N, K, Ap, sumA, Bp, sumB, zA, zB, C, ldc, stream);
    case 2: return launch_u4<FMT, 2, 2, 2, 2, S>(M, N, K, Ap, sumA, Bp, sumB, zA, zB, C, ldc, stream);
    default: return launch_u4<FMT, 2, 2, 1, 1, 4>(M, N, K, Ap, sumA, Bp, sumB, zA, zB, C, ldc, stream);
    }
}

// Shape-based choice.  256 x 256 tiles run one workgroup per compute unit, in rounds of 256 tiles; when the last round
// would be at most half full (784 tiles: 16 of them would run alone for a whole tile time), the columns of C that
// the full rounds cover go to one launch and the remaining columns to a second launch with 64 x 64 (or 128 x 128)
// tiles, which spreads them over the whole machine.  The packed right operand is ordered by row block, so a column
// range of C is a contiguous piece of it.
template <int FMT>
hipError_t launch_mx_auto(int64_t M, int64_t N, int64_t K, const uint8_t *Ap, const int32_t *sumA, const uint8_t *Bp,
                          const int32_t *sumB, int zA, int zB, int32_t *C, int64_t ldc, hipStream_t stream)
{
    const int forced = g_u4_forced.load(std::memory_order_relaxed);
    if (forced >= 0)
        return launch_mx_instance<FMT>(forced, M, N, K, Ap, sumA, Bp, sumB, zA, zB, C, ldc, stream);
    const int64_t nMB = (M + 255) / 256, nNB = (N + 255) / 256;
    const int64_t t256 = nMB * nNB, t128 = ((M + 127) / 128) * ((N + 127) / 128);
    const int inst = t256 >= 128 ? 1 : t128 >= 128 ? 2 : 3;
    const int64_t rest = t256 % kComputeUnits;
    if (inst == 1 && t256 > kComputeUnits && rest > 0 && rest <= kComputeUnits / 2) {
        const int64_t c1 = (t256 - rest) / nMB;  // whole columns of tiles inside the full rounds
        if (c1 >= 1 && c1 < nNB) {
            const int64_t N1 = c1 * 256, Nt = N - N1;
            const hipError_t e = launch_mx_instance<FMT>(1, M, N1, K, Ap, sumA, Bp, sumB, zA, zB, C, ldc, stream);
            if (e != hipSuccess)
                return e;
            constexpr int64_t kSeg = FMT == 2 ? 3072 : 2048;
            const int64_t t64 = ((M + 63) / 64) * ((Nt + 63) / 64);
            return launch_mx_instance<FMT>(t64 <= 4 * kComputeUnits ? 3 : 2, M, Nt, K, Ap, sumA,
                                           Bp + (N1 / 32) * ((K + 127) / 128) * kSeg, sumB ? sumB + N1 : nullptr, zA, zB,
                                           C + N1, ldc, stream);
        }
    }
    return launch_mx_instance<FMT>(inst, M, N, K, Ap, sumA, Bp, sumB, zA, zB, C, ldc, stream);
}

}  // namespace

int u4_num_instances() { return 4; }
void u4_force_instance(int t) { g_u4_forced.store(t, std::memory_order_relaxed); }

hipError_t launch_pack_u4(const uint8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k,
                          uint8_t *dst, int32_t *sums, hipStream_t stream)
{
    const int64_t RB = (rows + 31) / 32;
    const int KB = 2 * (int)((K + 127) / 128);
    if (RB > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, stream, sums, rows, 0);
    // about 4096 blocks at least, each looping over its share of the depth
    const int units = (KB * 2 + 7) / 8;
    int64_t chunks = (4096 + RB - 1) / RB;
    chunks = chunks < 1 ? 1 : chunks > units ? units : chunks;
    const dim3 grid((unsigned)RB, (unsigned)chunks);
    if (stride_k == 1) {
        hipLaunchKernelGGL(pack_u4_kernel, grid, dim3(256), 0, stream, src, rows, K, stride_r, dst, sums, KB);
    } else {
        const int64_t RB4 = (rows + 127) / 128;
        int64_t ch = (4096 + RB4 - 1) / RB4;
        ch = ch < 1 ? 1 : ch > units ? units : ch;
        hipLaunchKernelGGL(pack_u4_strided_kernel, dim3((unsigned)RB4, (unsigned)ch), dim3(256), 0, stream, src, rows, K,
                           stride_k, dst, sums, KB, RB);
    }
    return hipGetLastError();
}

hipError_t launch_gemm_u4(int64_t M, int64_t N, int64_t K, const uint8_t *Ap, const int32_t *sumA, const uint8_t *Bp,
                          const int32_t *sumB, int zA, int zB, int32_t *C, int64_t ldc, hipStream_t stream)
{
    return launch_mx_auto<2>(M, N, K, Ap, sumA, Bp, sumB, zA, zB, C, ldc, stream);
}

hipError_t launch_gemm_t4(int64_t M, int64_t N, int64_t K, const uint8_t *Ap, const uint8_t *Bp, int32_t *C, int64_t ldc,
                          hipStream_t stream)
{
    return launch_mx_auto<4>(M, N, K, Ap, nullptr, Bp, nullptr, 0, 0, C, ldc, stream);
}

hipError_t launch_pack_t4(const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, uint8_t *dst,
                          hipStream_t stream)
{
    const int64_t RB = (rows + 31) / 32;
    const int KB = 2 * (int)((K + 127) / 128);
    if (RB > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    const int units = (KB * 2 + 7) / 8;
    if (stride_k == 1) {
        int64_t chunks = (4096 + RB - 1) / RB;
        chunks = chunks < 1 ? 1 : chunks > units ? units : chunks;
        hipLaunchKernelGGL(pack_t4_kernel, dim3((unsigned)RB, (unsigned)chunks), dim3(256), 0, stream, src, rows, K,
                           stride_r, dst, KB);
    } else {
        const int64_t RB4 = (rows + 127) / 128;
        int64_t ch = (4096 + RB4 - 1) / RB4;
        ch = ch < 1 ? 1 : ch > units ? units : ch;
        hipLaunchKernelGGL(pack_t4_strided_kernel, dim3((unsigned)RB4, (unsigned)ch), dim3(256), 0, stream, src, rows, K,
                           stride_k, dst, KB, RB);
    }
    return hipGetLastError();
}

}  // namespace lowbit
