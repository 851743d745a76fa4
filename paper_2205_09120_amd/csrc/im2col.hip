// im2col in the packed domain: builds the packed right operand of a convolution-as-GEMM (one bit string per output
// pixel, depth order (ky, kx, channel); Section I and eq. (5) of the paper: depth = H_k * W_k * C_in) from a feature map
// that is already packed along its channels.  With the channel count a multiple of 64 every 64-bit depth word of
// the result is a verbatim copy of one word of one input pixel (or zero in the padding), so the lowering is a
// word gather: 9x less data is read than by unrolling the int8 map first, and each bit is encoded only once.
// HBM-bound: reads at most kh*kw times the packed map (mostly cache hits), writes the packed operand once.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lowbit_internal.h"

namespace lowbit {
namespace {

template <typename E> __device__ __forceinline__ E zero_e();
template <> __device__ __forceinline__ uint2 zero_e<uint2>() { return make_uint2(0u, 0u); }
template <> __device__ __forceinline__ uint4 zero_e<uint4>() { return make_uint4(0u, 0u, 0u, 0u); }

// One thread per output entry (pixel n, tap, channel word cw), cw fastest: stores are fully coalesced and the loads
// of one tap are CW consecutive entries of one input pixel.
template <typename E>
__global__ __launch_bounds__(256) void im2col_packed_kernel(const E *__restrict__ Fp, E *__restrict__ Bp, Im2colGeom g,
                                                            int64_t total)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total)
        return;
    const uint32_t kwout = (uint32_t)(g.kh * g.kw * g.CW);
    const int64_t n = idx / kwout;
    const uint32_t e = (uint32_t)(idx - n * kwout);
    const uint32_t tap = e / (uint32_t)g.CW, cw = e - tap * (uint32_t)g.CW;
    const int ky = (int)(tap / (uint32_t)g.kw), kx = (int)(tap - (uint32_t)ky * (uint32_t)g.kw);
    const int64_t plane = (int64_t)g.OH * g.OW;
    const int64_t b = n / plane;
    const uint32_t r = (uint32_t)(n - b * plane);
    const int oy = (int)(r / (uint32_t)g.OW), ox = (int)(r - (uint32_t)oy * (uint32_t)g.OW);
    const int iy = oy * g.sh + ky - g.ph, ix = ox * g.sw + kx - g.pw;
    E v = zero_e<E>();
    if (iy >= 0 && iy < g.H && ix >= 0 && ix < g.W)
        v = Fp[((b * g.H + iy) * g.W + ix) * g.CW + cw];
    Bp[idx] = v;
}

}  // namespace

hipError_t launch_im2col_packed(int planes, const uint64_t *Fp, uint64_t *Bp, const Im2colGeom &g, hipStream_t stream)
{
    const int64_t total = g.batch * g.OH * g.OW * (int64_t)g.kh * g.kw * g.CW;
    if (total == 0)
        return hipSuccess;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    if (planes == 2)
        hipLaunchKernelGGL(im2col_packed_kernel<uint4>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           reinterpret_cast<const uint4 *>(Fp), reinterpret_cast<uint4 *>(Bp), g, total);
    else
        hipLaunchKernelGGL(im2col_packed_kernel<uint2>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           reinterpret_cast<const uint2 *>(Fp), reinterpret_cast<uint2 *>(Bp), g, total);
    return hipGetLastError();
}

}  // namespace lowbit
