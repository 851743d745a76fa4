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

// One thread per 16-byte (8-byte) piece of the output: (pixel n, tap, piece u of the pixel's PW pieces), u fastest, so
// stores are fully coalesced and the loads of one tap are PW consecutive pieces of one input pixel.  A piece is one
// ternary entry, or two adjacent binary words when the channel word count is even (E = uint4), else one binary word
// (E = uint2).  I selects 32-bit index arithmetic when the piece count allows it: the integer divisions, not the
// memory system, bound this kernel otherwise.
template <typename E, typename I>
__global__ __launch_bounds__(256) void im2col_packed_kernel(const E *__restrict__ Fp, E *__restrict__ Bp, Im2colGeom g,
                                                            int PW, int64_t total)
{
    const int64_t idx64 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx64 >= total)
        return;
    const I idx = (I)idx64;
    const uint32_t per_pixel = (uint32_t)(g.kh * g.kw * PW);
    const I n = idx / (I)per_pixel;
    const uint32_t e = (uint32_t)(idx - n * (I)per_pixel);
    const uint32_t tap = e / (uint32_t)PW, u = e - tap * (uint32_t)PW;
    const int ky = (int)(tap / (uint32_t)g.kw), kx = (int)(tap - (uint32_t)ky * (uint32_t)g.kw);
    const I plane = (I)g.OH * (I)g.OW;
    const I b = n / plane;
    const uint32_t r = (uint32_t)(n - b * plane);
    const int oy = (int)(r / (uint32_t)g.OW), ox = (int)(r - (uint32_t)oy * (uint32_t)g.OW);
    const int iy = oy * g.sh + ky - g.ph, ix = ox * g.sw + kx - g.pw;
    E v = zero_e<E>();
    if (iy >= 0 && iy < g.H && ix >= 0 && ix < g.W)
        v = Fp[(((int64_t)b * g.H + iy) * g.W + ix) * PW + u];
    Bp[idx64] = v;
}

template <typename E>
hipError_t launch_pieces(const uint64_t *Fp, uint64_t *Bp, const Im2colGeom &g, int PW, hipStream_t stream)
{
    const int64_t total = g.batch * g.OH * g.OW * (int64_t)g.kh * g.kw * PW;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    const E *src = reinterpret_cast<const E *>(Fp);
    E *dst = reinterpret_cast<E *>(Bp);
    if (total < (int64_t)1 << 31)
        hipLaunchKernelGGL((im2col_packed_kernel<E, uint32_t>), dim3((unsigned)blocks), dim3(256), 0, stream, src, dst, g,
                           PW, total);
    else
        hipLaunchKernelGGL((im2col_packed_kernel<E, int64_t>), dim3((unsigned)blocks), dim3(256), 0, stream, src, dst, g,
                           PW, total);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_im2col_packed(int planes, const uint64_t *Fp, uint64_t *Bp, const Im2colGeom &g, hipStream_t stream)
{
    if (g.batch * g.OH * g.OW * (int64_t)g.kh * g.kw * g.CW == 0)
        return hipSuccess;
    if (planes == 2)
        return launch_pieces<uint4>(Fp, Bp, g, g.CW, stream);
    if (g.CW % 2 == 0)
        return launch_pieces<uint4>(Fp, Bp, g, g.CW / 2, stream);
    return launch_pieces<uint2>(Fp, Bp, g, g.CW, stream);
}

}  // namespace lowbit
