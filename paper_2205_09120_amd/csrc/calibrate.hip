// Calibration kernels for the benchmark: what this machine sustains for the two bounds the rooflines use.
//   * VALU: independent chains of exactly the instructions the GEMM kernels issue -- the binary pair (v_xor_b32,
//     v_bcnt_u32_b32 with accumulate) or the ternary four (v_and_b32, v_bitop3_b32 with a scalar source, two
//     v_bcnt_u32_b32) -- on registers, all wave slots occupied.  Counted work: threads * iters * 2 * CHAINS.
//   * HBM: streaming read (128-bit loads, XOR-reduced, one dword stored per thread), streaming write, and copy.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

constexpr int CHAINS = 16;

// MIX 0: the binary kernel's pair (xor, bcnt).  MIX 1: the ternary kernel's four (and, bitop3 with one scalar
// source, bcnt, bcnt).
template <int MIX>
__global__ __launch_bounds__(256) void calib_valu_kernel(int iters, uint32_t seed, uint32_t *__restrict__ sink)
{
    uint32_t a[CHAINS];
    int32_t acc[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) {
        a[c] = seed * (c + 1) + threadIdx.x;
        acc[c] = 0;
    }
    uint32_t b = seed ^ blockIdx.x;
    const uint32_t sb = __builtin_amdgcn_readfirstlane(b);
    int32_t acc2[CHAINS / 2];
#pragma unroll
    for (int c = 0; c < CHAINS / 2; ++c)
        acc2[c] = 0;
    for (int it = 0; it < iters; ++it) {
        if constexpr (MIX == 0) {
#pragma unroll
            for (int c = 0; c < CHAINS; ++c) {
                uint32_t x;
                asm volatile("v_xor_b32 %0, %1, %2" : "=v"(x) : "v"(a[c]), "v"(b));
                asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[c]) : "v"(x));
            }
        } else {
#pragma unroll
            for (int c = 0; c < CHAINS / 2; ++c) {
                uint32_t m, u;
                asm volatile("v_and_b32 %0, %1, %2" : "=v"(m) : "s"(sb), "v"(a[c]));
                asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x28" : "=v"(u) : "s"(sb), "v"(a[c + CHAINS / 2]), "v"(m));
                asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[c]) : "v"(m));
                asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc2[c]) : "v"(u));
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CHAINS / 2; ++c)
        acc[c] += acc2[c];
    int32_t s = 0;
#pragma unroll
    for (int c = 0; c < CHAINS; ++c)
        s += acc[c];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = (uint32_t)s;
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

int64_t calib_valu_lane_instr(int64_t iters) { return (int64_t)calib_grid_blocks() * 256 * iters * 2 * CHAINS; }

hipError_t launch_calib_valu(int mix, int iters, uint32_t *sink, hipStream_t stream)
{
    if (mix == 0)
        hipLaunchKernelGGL(calib_valu_kernel<0>, dim3(calib_grid_blocks()), dim3(256), 0, stream, iters, 0x9e3779b9u,
                           sink);
    else
        hipLaunchKernelGGL(calib_valu_kernel<1>, dim3(calib_grid_blocks()), dim3(256), 0, stream, iters, 0x9e3779b9u,
                           sink);
    return hipGetLastError();
}

hipError_t launch_calib_stream(int mode, const void *src, void *dst, int64_t bytes, uint32_t *sink, hipStream_t stream)
{
    const int64_t n16 = bytes / 16;
    const dim3 g(calib_grid_blocks() * 2), b(256);
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
