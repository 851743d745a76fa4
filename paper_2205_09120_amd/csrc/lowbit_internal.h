// Internal declarations shared by the HIP translation units of the library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lowbit {

#if defined(__HIPCC__)
// Result stores that write through the L2 of the XCD they are issued on (agent scope: the `sc1` bit of the store).
// A plain store leaves its line dirty in that L2 and the end of the kernel has to write all of them back before the
// next kernel on the stream may start -- time that nothing overlaps (measured on products that write 8 .. 50 MB:
// 1.5 - 2.7 us per launch, 3 - 8 % of kernels in the 30 - 60 us range).  Written through, the lines leave while the
// kernel is still computing.  Only for data the kernel does not read again, and only where a wave-wide store
// covers whole runs of a line (row-major C: 256 bytes per instruction); the packing kernels and the orientation
// where every lane stores to a line of its own measured equal or slower written through.
#ifndef LB_STORE_THROUGH
#define LB_STORE_THROUGH 1
#endif
__device__ __forceinline__ void store_through(int32_t *p, int32_t v)
{
#if LB_STORE_THROUGH
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#else
    *p = v;
#endif
}
// 16 bytes at any 4-byte aligned global address
__device__ __forceinline__ void store_through16(void *p, int32_t a, int32_t b, int32_t c, int32_t d)
{
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    const i32x4 q = {a, b, c, d};
#if LB_STORE_THROUGH
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(q) : "memory");
#else
    __builtin_memcpy(p, &q, 16);
#endif
}
#endif


// KIND_TBN_SV is the ternary-binary product with the TERNARY operand on the scalar side (launchers only: the C ABI
// knows kinds 0..2 and gemm_tbn picks the orientation).
enum Kind { KIND_BNN = 0, KIND_TNN = 1, KIND_TBN = 2, KIND_TBN_SV = 3 };

// One tiled popcount GEMM launch.  S is the scalar-side packed operand (rowsS bit strings), V the vector-side
// one (rowsV bit strings); product (s, v) is written to C[s*ldc + v], or to C[v*ldc + s] by the transposed
// launcher.  Operand classes per kind: BNN S,V binary; TNN S,V ternary; TBN S binary, V ternary; TBN_SV S ternary,
// V binary.
struct GemmArgs {
    const uint32_t *Sp;
    const uint32_t *Vp;
    int rowsS, rowsV, KW, K;
    int32_t *C;
    int64_t ldc;
    hipStream_t stream;
    int c16 = 0;  // 1: C is an int16_t matrix (ldc in 16-bit elements); the caller guarantees K <= 32767
    // Re-quantized output (transposed launcher only; q_out == nullptr selects the int32 store): instead of C, one
    // packed bit string per S row is written whose depth runs over the V rows, q_planes = 1 binary / 2 ternary,
    // thresholds per V row.
    const int32_t *q_lo = nullptr;
    const int32_t *q_hi = nullptr;
    uint64_t *q_out = nullptr;
    int q_planes = 0;
};

struct Im2colGeom;

struct GemmVariant {
    const char *name;
    int rank;          // preference of the shape-based selection, 0 = manual only
    int tileS, tileV;  // workgroup tile extents along S and V
    hipError_t (*launch)(const GemmArgs &);
    hipError_t (*launch_transposed)(const GemmArgs &);
    int small_max;     // > 0: chosen for problems of at most this many 16 x 64 tiles (first match in table order) ...
    int small_min_kw;  // ... whose depth is at least this many 64-bit words (ranked variants: taken only from this depth on)
    // the same instance with the V operand gathered from a channel-packed feature map (convolution without the
    // unrolled operand; a.Vp is the packed map, a.rowsV the output pixels); hipErrorNotSupported for the kinds whose
    // gathered operand would sit on the scalar side
    hipError_t (*launch_conv)(const GemmArgs &, const Im2colGeom &);
    int wanted_wg = 0;  // ranked variants: workgroups the problem must yield (0: the selection's default for the rank)
};

const GemmVariant *gemm_variants(int kind, int *count);

// Depth-split launch of the 8 x 64 instance for products of few tiles and a long depth: clears C (int32 only), then
// adds the partial products of `nsplit` depth ranges with integer atomics.  Two kernels on a.stream.
hipError_t launch_gemm_splitk(int kind, const GemmArgs &a, bool transposed, int nsplit);

// Grouped launch: one grid covers `count` independent problems, each cut into kGroupTileS x kGroupTileV tiles.
// The table is header, `count` records, then one uint32 per workgroup naming the record that owns it; it is built on
// the host (api.hip), copied to the device by the caller and read by the kernel.
constexpr int kGroupTileS = 16, kGroupTileV = 64;
constexpr uint32_t kGroupMagic = 0x4c424754u;  // "LBGT"
struct GroupHeader {
    uint32_t magic;
    uint32_t kind;
    uint32_t count;
    uint32_t workgroups;
};
struct GroupRecord {
    const uint32_t *Sp;  // scalar-side operand, rowsS strings
    const uint32_t *Vp;  // vector-side operand, rowsV strings
    int32_t *C;
    int64_t ldc;
    int32_t rowsS, rowsV, KW, K;
    int32_t nSB;         // tiles along S; tile t of the problem is (vb, sb) = (t / nSB, t % nSB)
    uint32_t tile0;      // first workgroup of the problem
    int32_t transposed;  // 0: product (s, v) -> C[s*ldc + v]; 1: -> C[v*ldc + s]
    int32_t reserved;
};
static_assert(sizeof(GroupHeader) == 16 && sizeof(GroupRecord) == 64, "table layout is part of the host/device contract");
hipError_t launch_gemm_group(int kind, const GroupHeader *table_dev, uint32_t count, uint32_t workgroups,
                             hipStream_t stream);
// The same launch with the table in the library's own per-device array instead of caller memory: the HOST table is
// uploaded in pieces of kGroupChunkBytes through kernel arguments (no allocation, no memcpy call), then the group
// kernel runs on it.  table_bytes must be a positive multiple of 16 and at most kGroupStaticBytes.
constexpr size_t kGroupStaticBytes = 64 * 1024;
constexpr size_t kGroupChunkBytes = 3584;
hipError_t launch_gemm_group_static(int kind, const void *table_host, size_t table_bytes, uint32_t count,
                                    uint32_t workgroups, hipStream_t stream);

// Skinny launch (gemm_skinny.hip): X is the large streamed operand, Y the small one (any count; processed 8, 16 or
// 32 strings at a time: X is streamed once for up to 32).  Product (x, y) goes to C[x*ldc + y], or C[y*ldc + x] when transposed.
// Operand classes per kind: BNN X,Y binary; TNN X,Y ternary; TBN X ternary, Y binary; TBN_SV X binary, Y ternary.
struct SkinnyArgs {
    const void *Xp;
    const void *Yp;
    int rowsX, rowsY, KW, K;
    int32_t *C;
    int64_t ldc;
    hipStream_t stream;
    int c16 = 0;  // as in GemmArgs
};
hipError_t launch_gemm_skinny(int kind, const SkinnyArgs &a, bool transposed);
int skinny_num_configs();
void skinny_force_config(int cfg);  // -1 = shape-based
int skinny_forced_config();

// Packing launchers (pack.hip).  Element (r,k) = src[r*stride_r + k*stride_k].
hipError_t launch_pack(bool ternary, const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k,
                       uint64_t *dst, hipStream_t stream);

// Packed-domain im2col (im2col.hip).  CW = channel words (C/64); OH, OW are the output map extents.
struct Im2colGeom {
    int64_t batch;
    int H, W, CW, OH, OW;
    int kh, kw, sh, sw, ph, pw;
};
hipError_t launch_im2col_packed(int planes, const uint64_t *Fp, uint64_t *Bp, const Im2colGeom &g, hipStream_t stream);

// Calibration kernels (calibrate.hip).  sink needs calib_grid_blocks()*2*256 dwords (mode 0 of the stream kernel:
// blocks*256 dwords when a grid size is given).
// VALU instruction mixes: the three kernels' own (binary, ternary, ternary-binary) and single instruction forms.
enum CalibMix { CALIB_BNN = 0, CALIB_TNN = 1, CALIB_TBN = 2, CALIB_XOR_VV = 3, CALIB_AND_SV = 4, CALIB_BITOP_SVV = 5,
                CALIB_BCNT = 6, CALIB_NUM_MIXES = 7 };
int calib_grid_blocks();
int64_t calib_valu_lane_instr(int mix, int64_t iters, int waves_per_simd);
// clocks: nullptr, or 2 x 256 x waves_per_simd 64-bit values: per workgroup the ticks of the shader-clock counter and
// of the constant-rate counter (calib_wall_clock_khz() ticks per millisecond) that passed while its first wave ran
hipError_t launch_calib_valu(int mix, int iters, int waves_per_simd, uint32_t *sink, unsigned long long *clocks,
                             hipStream_t stream);
int calib_wall_clock_khz();  // 0 if the runtime does not report it
// blocks: grid size of the streaming kernel (workgroups of 256 threads), 0 = the default of 16 per compute unit
hipError_t launch_calib_stream(int mode, const void *src, void *dst, int64_t bytes, int blocks, uint32_t *sink,
                               hipStream_t stream);

// int8 matrix-core GEMM launcher (gemm_i8_mfma.hip).
hipError_t launch_gemm_i8(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                          int32_t *C, int64_t ldc, hipStream_t stream);
hipError_t launch_gemm_u8(int64_t M, int64_t N, int64_t K, const uint8_t *A, int64_t lda, const uint8_t *B, int64_t ldb,
                          int zA, int zB, int32_t *C, int64_t ldc, hipStream_t stream);
hipError_t launch_gemm_i8_skinny(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B,
                                 int64_t ldb, int32_t *C, int64_t ldc, hipStream_t stream);
// Grouped launch of the comparator: 64 x 64 tiles (the instance small products take), table = header, `count` records,
// one uint32 per workgroup naming its record; built on the host (api.hip), copied to the device by the caller.
constexpr int kI8GroupTile = 64;
constexpr uint32_t kI8GroupMagic = 0x4c423847u;  // "LB8G"
struct I8GroupHeader {
    uint32_t magic, count, workgroups, reserved;
};
struct I8GroupRecord {
    const int8_t *A;
    const int8_t *B;
    int32_t *C;
    int64_t lda, ldb, ldc;
    int32_t M, N, K;
    int32_t nMB;     // tiles along M; tile t of the problem is (nb, mb) = (t / nMB, t % nMB)
    uint32_t tile0;  // first workgroup of the problem
    int32_t mode;    // fetch mode (i8_fetch_mode)
    int32_t reserved[2];
};
static_assert(sizeof(I8GroupHeader) == 16 && sizeof(I8GroupRecord) == 80, "table layout is part of the host/device contract");
int i8_fetch_mode(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb, int BM, int BN);
hipError_t launch_gemm_i8_group(const I8GroupHeader *table_dev, uint32_t count, uint32_t workgroups, hipStream_t stream);
void i8_force_tile(int t);  // -1 = shape-based, 0 = 128x128, 1 = 256x256, 2 = 256x128 (4 waves each),
                            // 3 / 4 / 5 = wave-specialised 256x128 with 3 / 2 / 4 depth steps of prefetch,
                            // 6 = direct-to-LDS 256x128 with 4 stages of 64 depth bytes, 7 / 8 / 9 = direct-to-LDS
                            // 256x128 / 128x128 / 64x64 with 3 stages of 128 depth bytes (4 of 64 if the depth is
                            // not a multiple of 128); ragged extents allowed

// 4-bit unsigned operands as 6-bit floats on the scaled matrix-core instruction (gemm_mx_mfma.hip).  Packed operands
// are fragment-major (see that file); sums holds one int32 per row.  Element (r,k) = src[r*stride_r + k*stride_k].
hipError_t launch_pack_u4(const uint8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k,
                          uint8_t *dst, int32_t *sums, hipStream_t stream);
hipError_t launch_gemm_u4(int64_t M, int64_t N, int64_t K, const uint8_t *Ap, const int32_t *sumA, const uint8_t *Bp,
                          const int32_t *sumB, int zA, int zB, int32_t *C, int64_t ldc, hipStream_t stream);
// The same kernel on ternary / binary operands stored as 4-bit floats (no sums, no zero points).
hipError_t launch_pack_t4(const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, uint8_t *dst,
                          hipStream_t stream);
hipError_t launch_gemm_t4(int64_t M, int64_t N, int64_t K, const uint8_t *Ap, const uint8_t *Bp, int32_t *C, int64_t ldc,
                          hipStream_t stream);
int u4_num_instances();
void u4_force_instance(int t);  // -1 = shape-based

}  // namespace lowbit
