// Calibration kernels for the benchmark: what this machine sustains for the two bounds the rooflines use.
//   * VALU: independent chains, on registers only, of exactly the instruction forms the GEMM kernels issue per
//     32 depth positions and output -- binary: v_xor_b32 with a scalar source + v_bcnt_u32_b32 (accumulating);
//     ternary: v_and_b32 with a scalar source, v_bitop3_b32 with one scalar source, two v_bcnt_u32_b32;
//     ternary-binary: v_bitop3_b32 with one scalar source + v_bcnt_u32_b32 -- and of single instruction forms, with
//     1 .. 8 waves on every SIMD.  The rate of a mix is NOT 64 lanes per clock and compute unit for every form:
//     two-source logic on vector registers issues at up to 1.7x that, three-source forms and popcounts at 0.9x, and a
//     mix lands in between, so the ceiling of a kernel is the rate its own mix reaches here.
//     Each workgroup also reports the engine clock it ran at (shader-clock ticks against constant-rate ticks).
//   * HBM: streaming read (128-bit loads, XOR-reduced, one dword stored per thread), streaming write, and copy.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

constexpr int CHAINS = 8;

#define LB_AND_SV(m, s, a) asm volatile("v_and_b32 %0, %1, %2" : "=v"(m) : "s"(s), "v"(a))
#define LB_XOR_SV(m, s, a) asm volatile("v_xor_b32 %0, %1, %2" : "=v"(m) : "s"(s), "v"(a))
#define LB_XOR_VV(m, a, b) asm volatile("v_xor_b32 %0, %1, %2" : "=v"(m) : "v"(a), "v"(b))
#define LB_BITOP_SVV(u, s, b, m) asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x28" : "=v"(u) : "s"(s), "v"(b), "v"(m))
#define LB_BCNT(acc, x) asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x))

// lane-instructions one loop iteration of a mix issues per thread
__host__ __device__ constexpr int calib_per_iter(int mix)
{
    return mix == CALIB_TNN ? 4 * CHAINS : (mix == CALIB_BNN || mix == CALIB_TBN) ? 2 * CHAINS : CHAINS;
}

template <int MIX>
__global__ __launch_bounds__(256) void calib_valu_kernel(int iters, uint32_t seed, uint32_t *__restrict__ sink,
                                                         unsigned long long *__restrict__ clocks)
{
    uint32_t a[CHAINS], b[CHAINS], s[CHAINS], m[CHAINS], u[CHAINS];
    int32_t acc[CHAINS], acc2[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) {
        a[c] = seed * (c + 1) + threadIdx.x;
        b[c] = a[c] * 7u + 3u;
        m[c] = u[c] = 0;
        acc[c] = acc2[c] = 0;
        s[c] = __builtin_amdgcn_readfirstlane((seed >> c) ^ (blockIdx.x * (c + 3)));
    }
    // shader-clock counter (advances with the engine clock) and constant-rate counter, read around the chain: their
    // ratio is the engine clock this wave ran at
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        if constexpr (MIX == CALIB_BNN) {
#pragma unroll
            for (int c = 0; c < CHAINS; ++c) {
                LB_XOR_SV(m[c], s[c], a[c]);
                LB_BCNT(acc[c], m[c]);
            }
        } else if constexpr (MIX == CALIB_TNN) {
            // the four instructions of one unit, two units in flight so that no instruction waits for the one before
            // it (measured: 4-6 % faster than issuing each unit's four back to back)
            LB_AND_SV(m[0], s[0], a[0]);
            LB_BITOP_SVV(u[0], s[1], b[0], m[0]);
#pragma unroll
            for (int c = 0; c < CHAINS; ++c) {
                LB_BCNT(acc[c], m[c]);
                if (c + 1 < CHAINS)
                    LB_AND_SV(m[c + 1], s[c + 1], a[c + 1]);
                LB_BCNT(acc2[c], u[c]);
                if (c + 1 < CHAINS)
                    LB_BITOP_SVV(u[c + 1], s[(c + 2) % CHAINS], b[c + 1], m[c + 1]);
            }
        } else if constexpr (MIX == CALIB_TBN) {
#pragma unroll
            for (int c = 0; c < CHAINS; ++c) {
                LB_BITOP_SVV(u[c], s[c], b[c], a[c]);
                LB_BCNT(acc[c], u[c]);
            }
        } else if constexpr (MIX == CALIB_XOR_VV) {
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
                LB_XOR_VV(m[c], a[c], b[c]);
        } else if constexpr (MIX == CALIB_AND_SV) {
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
                LB_AND_SV(m[c], s[c], a[c]);
        } else if constexpr (MIX == CALIB_BITOP_SVV) {
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
                LB_BITOP_SVV(u[c], s[c], b[c], a[c]);
        } else {
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
                LB_BCNT(acc[c], a[c]);
        }
    }
    // the popcount sums are the result (checkable on the host); forms without a count keep their last values alive
    int32_t r = 0;
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) {
        r += acc[c] + acc2[c];
        if constexpr (MIX == CALIB_XOR_VV || MIX == CALIB_AND_SV || MIX == CALIB_BITOP_SVV)
            r += (int32_t)(m[c] ^ u[c]);
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = (uint32_t)r;
    // the reads below depend on r, so they cannot move above the chain
    if (clocks != nullptr && threadIdx.x == 0) {
        unsigned long long c1 = clock64(), w1 = wall_clock64();
        if (r == 0x7fffffff)
            c1 += 1;
        clocks[(size_t)blockIdx.x * 2] = c1 - c0;
        clocks[(size_t)blockIdx.x * 2 + 1] = w1 - w0;
    }
}

__global__ __launch_bounds__(256) void calib_read_kernel(const uint4 *__restrict__ src, int64_t n16,
                                                         uint32_t *__restrict__ sink)
{
    uint4 s = make_uint4(0u, 0u, 0u, 0u);
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const uint4 v = src[i];
        s.x ^= v.x;
        s.y ^= v.y;
        s.z ^= v.z;
        s.w ^= v.w;
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s.x ^ s.y ^ s.z ^ s.w;
}

__global__ __launch_bounds__(256) void calib_write_kernel(uint4 *__restrict__ dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const uint4 v = make_uint4(1u, 2u, 3u, 4u);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        dst[i] = v;
}

__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                         int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

}  // namespace

int calib_grid_blocks() { return 256 * 8; }  // 8 workgroups of 4 waves per compute unit: every wave slot busy

int64_t calib_valu_lane_instr(int mix, int64_t iters, int waves_per_simd)
{
    return (int64_t)256 * waves_per_simd * 256 * iters * calib_per_iter(mix);
}

hipError_t launch_calib_valu(int mix, int iters, int waves_per_simd, uint32_t *sink, unsigned long long *clocks,
                             hipStream_t stream)
{
    // one workgroup of 4 waves per compute unit and wave slot wanted (256 compute units)
    const dim3 grid(256 * waves_per_simd), block(256);
    const uint32_t seed = 0x9e3779b9u;
    switch (mix) {
    case CALIB_BNN: hipLaunchKernelGGL(calib_valu_kernel<CALIB_BNN>, grid, block, 0, stream, iters, seed, sink, clocks); break;
    case CALIB_TNN: hipLaunchKernelGGL(calib_valu_kernel<CALIB_TNN>, grid, block, 0, stream, iters, seed, sink, clocks); break;
    case CALIB_TBN: hipLaunchKernelGGL(calib_valu_kernel<CALIB_TBN>, grid, block, 0, stream, iters, seed, sink, clocks); break;
    case CALIB_XOR_VV: hipLaunchKernelGGL(calib_valu_kernel<CALIB_XOR_VV>, grid, block, 0, stream, iters, seed, sink, clocks); break;
    case CALIB_AND_SV: hipLaunchKernelGGL(calib_valu_kernel<CALIB_AND_SV>, grid, block, 0, stream, iters, seed, sink, clocks); break;
    case CALIB_BITOP_SVV: hipLaunchKernelGGL(calib_valu_kernel<CALIB_BITOP_SVV>, grid, block, 0, stream, iters, seed, sink, clocks); break;
    case CALIB_BCNT: hipLaunchKernelGGL(calib_valu_kernel<CALIB_BCNT>, grid, block, 0, stream, iters, seed, sink, clocks); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

int calib_wall_clock_khz()
{
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess)
        return 0;
    return khz;
}

hipError_t launch_calib_stream(int mode, const void *src, void *dst, int64_t bytes, int blocks, uint32_t *sink,
                               hipStream_t stream)
{
    const int64_t n16 = bytes / 16;
    const dim3 g(blocks > 0 ? blocks : calib_grid_blocks() * 2), b(256);
    if (mode == 0)
        hipLaunchKernelGGL(calib_read_kernel, g, b, 0, stream, static_cast<const uint4 *>(src), n16, sink);
    else if (mode == 1)
        hipLaunchKernelGGL(calib_write_kernel, g, b, 0, stream, static_cast<uint4 *>(dst), n16);
    else
        hipLaunchKernelGGL(calib_copy_kernel, g, b, 0, stream, static_cast<const uint4 *>(src),
                           static_cast<uint4 *>(dst), n16);
    return hipGetLastError();
}

}  // namespace lowbit
