/*
 * lowbit_gemm_bench.h -- hooks of liblowbit_gemm.so for benchmarks and tuning runs only: calibration kernels for the
 * two roofline bounds and a switch that forces a kernel variant.  Not part of the product boundary (lowbit_gemm.h);
 * same calling rules (device pointers, `stream` a hipStream_t passed as void*, lb_status return values).
 */
#ifndef LOWBIT_GEMM_BENCH_H
#define LOWBIT_GEMM_BENCH_H

#include "lowbit_gemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Calibration kernels for the benchmark: what the machine sustains for the two bounds of the rooflines.  The
 * caller times them (HIP events on `stream`).
 *   lb_calib_valu     runs lb_calib_valu_lane_instr(mix, iters, waves_per_simd) lane-instructions of independent
 *                     chains on registers, waves_per_simd (1..8) waves on every SIMD of the device, iters in
 *                     [1, 2^24] (the count is 0 for arguments outside these ranges).  mix 0: the binary
 *                     kernel's pair (v_xor_b32 with a scalar source, v_bcnt_u32_b32), 1: the ternary kernel's four
 *                     (v_and_b32 and v_bitop3_b32 with a scalar source, 2 x v_bcnt_u32_b32), 2: the ternary-binary
 *                     kernel's pair (v_bitop3_b32 with a scalar source, v_bcnt_u32_b32); single instruction forms:
 *                     3 v_xor_b32 on two vector registers, 4 v_and_b32 with a scalar source, 5 v_bitop3_b32 with a
 *                     scalar source, 6 v_bcnt_u32_b32.
 *   lb_calib_stream   mode 0: read `bytes` from src; 1: write `bytes` to dst; 2: copy src -> dst (128-bit accesses,
 *                     bytes a multiple of 16; src / dst may be NULL for the mode that does not use them); blocks =
 *                     workgroups of 256 threads in the grid (0: 16 per compute unit; at most 4096).
 *   sink              device scratch owned by the caller, at least lb_calib_sink_bytes() bytes; receives per-thread
 *                     results so that the work cannot be optimized away.
 *   clocks            NULL, or device memory of lb_calib_clocks_bytes() bytes: per workgroup (256 x waves_per_simd of
 *                     them) two uint64, the ticks of the shader-clock counter and of the constant-rate counter
 *                     (lb_calib_wall_clock_khz() ticks per millisecond; 0 if the runtime does not report it) that
 *                     passed while the workgroup's first wave ran its chain.  shader ticks / constant ticks * that
 *                     rate = the engine clock under this load.
 */
LB_API size_t lb_calib_sink_bytes(void);
LB_API size_t lb_calib_clocks_bytes(void);
LB_API int lb_calib_wall_clock_khz(void);
LB_API int64_t lb_calib_valu_lane_instr(int mix, int64_t iters, int waves_per_simd);
LB_API int lb_calib_valu(int mix, int64_t iters, int waves_per_simd, void *sink, void *clocks, void *stream);
LB_API int lb_calib_stream(int mode, const void *src, void *dst, int64_t bytes, int blocks, void *sink, void *stream);

/*
 * Tuning hook for benchmarks: force the tile variant used by one of the gemm_* entry points.
 *   op       0 = gemm_bnn, 1 = gemm_tnn, 2 = gemm_tbn (tile variant of the tiled kernel; forcing one also keeps
 *            skinny problems on the tiled kernel), 3 = configuration of the skinny (depth-split) kernel (forcing one
 *            also sends every product with at most 32 strings on one side to that kernel),
 *            4 = kernel instance of gemm_i8_mfma (0..2: 4-wave tiles 128x128, 256x256, 256x128; 3..5: wave-specialised
 *            256x128 with 3, 2, 4 depth steps of prefetch; 6: direct-to-LDS 256x128 with 64-byte depth stages;
 *            7, 8, 9: direct-to-LDS 256x128 / 128x128 / 64x64 tiles with 128-byte stages where the depth allows;
 *            an instance that cannot serve a shape falls back to the next simpler one),
 *            5 = kernel instance of gemm_u4_mfma and gemm_t4_mfma (0: 256x256 tile with 4 waves, 1: 256x256 with 8
 *            waves, 2: 128x128, 3: 64x64)
 *   variant  index into that op's variant table, or -1 to restore shape-based selection.
 * Returns LB_OK, or LB_EINVAL if op/variant is out of range.  lb_num_variants(op) gives the table size and
 * lb_variant_name(op, variant) a short description (host string owned by the library, NULL if out of range).
 * Process-wide (atomic integers, read once per call): a change made while other threads are inside gemm_* calls
 * affects the calls that start after it.
 */
LB_API int lb_set_variant(int op, int variant);

LB_API int lb_num_variants(int op);
LB_API const char *lb_variant_name(int op, int variant);

#ifdef __cplusplus
}
#endif
#endif /* LOWBIT_GEMM_BENCH_H */
