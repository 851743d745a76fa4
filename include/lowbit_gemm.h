/*
 * lowbit_gemm.h -- C ABI of the MI355X (gfx950) low-bit matrix multiplication library.
 *
 * The library computes C = A B (A: M x K, B: K x N, C: M x N, the "height", "width" and
 * "depth" of Section II-A of the paper) for the three operand classes of Section III:
 *     BNN  A, B in {-1,+1}
 *     TNN  A, B in {-1,0,+1}
 *     TBN  A in {-1,0,+1}, B in {-1,+1}
 * on bit-packed operands (Section III-A): a binary value is one bit (+1 -> 0, -1 -> 1), a
 * ternary value two bits (x+, x-) with +1 -> (1,0), 0 -> (0,0), -1 -> (0,1); the product is
 * obtained with AND/OR/XOR and population counts (eq. (6) and (7)).  Results are exact.
 * The paper accumulates in signed 16-bit lanes (k_max = 32767, Section IV-A); this library
 * accumulates and stores 32-bit integers, which gives the same values for every K the paper
 * allows and lifts the depth limit to 2^31 - 1.
 *
 * General rules for every entry point
 *   - Every pointer argument is a DEVICE pointer on the current HIP device, owned by the
 *     caller, and must stay valid until the work queued on `stream` has finished.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work: they do not synchronize, do not allocate and do not free.
 *   - Return value: LB_OK (0) or a negative lb_status.  On failure nothing was enqueued
 *     (except LB_EHIP, where the runtime refused a launch) and lb_last_error() returns a
 *     message for the calling thread.
 *   - Pointers must be aligned to 16 bytes (packed operands, int8 sources) or 4 bytes (C).
 *
 * Packed operand format (version LB_FORMAT_VERSION)
 *   A matrix is packed as `rows` bit strings along the depth k; KW = ceil(K/64).
 *   Word w of a bit string holds depth positions 64w .. 64w+63, position k in bit (k mod 64)
 *   counted from the least significant bit.  Little-endian uint64_t.
 *     binary :  dst[r*KW + w]
 *     ternary:  dst[(r*KW + w)*2 + 0] = plus plane (x+),  dst[(r*KW + w)*2 + 1] = minus plane (x-)
 *   Positions k >= K in the last word are 0 in every plane.
 *   For A (M x K) the bit strings are its rows; for B (K x N) they are its columns.
 */
#ifndef LOWBIT_GEMM_H
#define LOWBIT_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LB_FORMAT_VERSION 1

#if defined(__GNUC__)
#define LB_API __attribute__((visibility("default")))
#else
#define LB_API
#endif

typedef enum lb_status {
    LB_OK = 0,
    LB_EINVAL = -1,       /* null pointer, non-positive dimension, bad stride / leading dimension, misaligned pointer */
    LB_EOVERFLOW = -2,    /* a size does not fit the index arithmetic (K > 2^31-1, rows*KW too large, ...) */
    LB_EHIP = -3,         /* the HIP runtime reported an error at launch; message holds hipGetErrorString */
    LB_EUNSUPPORTED = -4  /* valid request that this build cannot serve (e.g. device is not gfx950) */
} lb_status;

/* Message describing the last failure on the calling thread ("" if none).  Host pointer, owned by the library. */
LB_API const char *lb_last_error(void);

/* LB_FORMAT_VERSION the library was built with. */
LB_API int lb_format_version(void);

/* 1 if a device with this architecture name (hipDeviceProp_t::gcnArchName, e.g. "gfx950:sramecc+:xnack-") can run
 * the library, else 0.  The library holds gfx950 machine code only; on any other device every entry point that would
 * launch a kernel returns LB_EUNSUPPORTED instead (checked once per device).  Host logic, usable without a GPU. */
LB_API int lb_arch_supported(const char *gcn_arch_name);

/* Bytes of a packed operand of `rows` bit strings of depth K: rows*ceil(K/64)*8 (binary) or *16 (ternary).
 * Returns 0 when rows < 0, K < 0 or the size overflows size_t. */
LB_API size_t packed_binary_bytes(int64_t rows, int64_t K);
LB_API size_t packed_ternary_bytes(int64_t rows, int64_t K);

/*
 * pack_binary / pack_ternary -- encode an int8 matrix into the packed format (Section III-A encodings;
 * they take the place of the paper's PackNRowsA / PackNColsB reorder step of Algorithms 1 and 2).
 *
 *   src       device, int8.  Element (r, k) of the `rows` x K logical matrix is src[r*stride_r + k*stride_k].
 *             A (M x K row-major): rows = M, stride_r = lda (>= K), stride_k = 1.
 *             B (K x N row-major): rows = N, stride_r = 1, stride_k = ldb (>= N).
 *             One of the two strides must be 1 and the other >= the extent it strides over.
 *   dst       device, packed_*_bytes(rows, K) bytes, overwritten completely (pad bits included).
 *   Encoding  binary:  x < 0 -> bit 1, otherwise bit 0.
 *             ternary: x > 0 -> (1,0), x < 0 -> (0,1), x == 0 -> (0,0).  The code (1,1) is never produced.
 *             Inputs outside the legal value sets are encoded by sign as above; no error is raised.
 * rows == 0 or K == 0 is a valid no-op.
 */
LB_API int pack_binary(const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, uint64_t *dst,
                void *stream);
LB_API int pack_ternary(const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, uint64_t *dst,
                 void *stream);

/*
 * im2col_packed -- lower a convolution to the GEMM above without unrolling the int8 feature map: gather the packed
 * right operand (one bit string per output pixel) from a feature map that is already packed along its channels.
 * The paper computes convolutions as matrix products after an im2col unrolling (Section I; Section IV-A and eq. (5):
 * depth = H_k * W_k * C_in); this call does that unrolling on packed words.
 *
 *   Fp        device, packed feature map: batch*H*W bit strings (pixels in NHWC order) of depth C, i.e. the output of
 *             pack_binary / pack_ternary(fmap, rows = batch*H*W, K = C, stride_r = C, stride_k = 1).
 *   planes    1 = binary strings, 2 = ternary strings (plus and minus word adjacent).
 *   C         channels; must be a multiple of 64 (LB_EUNSUPPORTED otherwise: unroll the int8 map and use pack_*).
 *   kh, kw    window; stride_h/w >= 1; pad_h/w >= 0 (padding with zero WORDS, see Bp).
 *   Bp        device, out: N = batch*OH*OW bit strings of depth K = kh*kw*C with OH = (H + 2*pad_h - kh)/stride_h + 1,
 *             OW likewise; string n = (b*OH + oy)*OW + ox; depth index (ky*kw + kx)*C + c.  Size
 *             packed_binary_bytes(N, K) or packed_ternary_bytes(N, K).  Positions in the padding are zero words:
 *             the ternary value 0, or the binary value +1 (a binary map cannot represent 0).
 * The matching left operand holds one filter per row with the same (ky, kx, c) depth order.
 * An empty problem (batch == 0, or a window larger than the padded map) is a valid no-op.
 */
LB_API int im2col_packed(const uint64_t *Fp, int planes, int64_t batch, int64_t H, int64_t W, int64_t C, int kh, int kw,
                         int stride_h, int stride_w, int pad_h, int pad_w, uint64_t *Bp, void *stream);

/*
 * conv_gemm -- a convolution layer as one call: C = A * im2col(feature map), with the unrolled operand never written.
 * The product kernel gathers the packed words of the right operand (depth order (ky, kx, c), eq. (5)) from the
 * channel-packed feature map while it stages its tiles; the values written are those of im2col_packed followed by
 * gemm_bnn / gemm_tnn.
 *
 *   kind      0 = BNN (binary filters, binary map), 1 = TNN (ternary filters, ternary map).  2 (TBN) is
 *             LB_EUNSUPPORTED: that kernel keeps the binary operand in scalar registers; use im2col_packed + gemm_tbn.
 *   Ap        device, packed filters: M strings of depth K = kh*kw*C in (ky, kx, c) order
 *   Fp        device, packed feature map as for im2col_packed (batch*H*W strings of depth C, C a multiple of 64)
 *   C         device, int32 row-major M x N with N = batch*OH*OW (string n = (b*OH + oy)*OW + ox), ldc >= N; overwritten
 *   padding   positions outside the map contribute zero words: the ternary value 0, or the binary value +1
 * Geometry rules and errors as for im2col_packed and gemm_*; an empty problem is a valid no-op.
 */
LB_API int conv_gemm(int kind, int64_t M, const uint64_t *Ap, const uint64_t *Fp, int64_t batch, int64_t H, int64_t W,
                     int64_t C, int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w, int32_t *Cout,
                     int64_t ldc, void *stream);

/*
 * gemm_bnn -- binary x binary, eq. (6):  C[i][j] = K - 2 * sum_w popcount(Ap[i][w] xor Bp[j][w]).
 * gemm_tnn -- ternary x ternary, eq. (7) with the ternary product of Section III-A (Table I, columns z+, z-).
 * gemm_tbn -- ternary A x binary B, eq. (7) with the ternary-binary product (Table I, columns u+, u-).
 *
 *   Ap        device, packed A: M bit strings of depth K (binary for gemm_bnn, ternary otherwise).
 *   Bp        device, packed B: N bit strings (the columns of B) of depth K (ternary for gemm_tnn, binary otherwise).
 *   C         device, int32, row-major M x N with leading dimension ldc >= N; overwritten (no accumulation into C;
 *             its previous contents do not matter).  A call enqueues one kernel, or two for products of few tiles
 *             and a long depth (C is cleared, then partial products of depth ranges are added with integer atomics):
 *             C holds the result once the work enqueued by the call has completed, not before.
 *   K         true depth (pad bits of the last word must be 0 as pack_* writes them); 1 <= K <= 2^31 - 1.
 * The kernels evaluate algebraically equivalent forms of the paper's bit formulas (see the kernel sources);
 * the integers written are identical.  Packed operands holding the invalid ternary code (1,1) give undefined C.
 * M == 0 or N == 0 is a valid no-op; K == 0 is LB_EINVAL.
 */
LB_API int gemm_bnn(int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp, int32_t *C, int64_t ldc,
             void *stream);
LB_API int gemm_tnn(int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp, int32_t *C, int64_t ldc,
             void *stream);
LB_API int gemm_tbn(int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp, int32_t *C, int64_t ldc,
             void *stream);

/*
 * gemm_c16 -- gemm_bnn / gemm_tnn / gemm_tbn writing a signed 16-bit C, the accumulator and output width of the
 * paper's microkernels (Section III; Table II, k_max = 32767 for all three).  Since |c| <= K, the values are the ones
 * the int32 calls write whenever K <= 32767; the C store, which dominates the traffic of shallow products, is halved.
 *
 *   kind   0 = BNN, 1 = TNN, 2 = TBN operands (Ap, Bp as for the corresponding gemm_* call)
 *   C      device, int16, row-major M x N with leading dimension ldc >= N (in 16-bit elements), 2-byte aligned;
 *          overwritten.
 *   K      1 <= K <= 32767; a larger depth is LB_EOVERFLOW (eq. (4) with a signed 16-bit result).
 * Everything else as for gemm_bnn / gemm_tnn / gemm_tbn.
 */
LB_API int gemm_c16(int kind, int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp, int16_t *C,
                    int64_t ldc, void *stream);

/*
 * gemm_requant -- gemm_bnn / gemm_tnn / gemm_tbn with the activation threshold fused into the epilogue: instead of
 * the int32 matrix C the call writes the low-bit feature map the next layer consumes, already packed.  The paper's
 * algorithms stop at the integer C (Section III); this is the step that follows it in a BNN / TNN / TBN layer.
 *
 *   kind        0 = BNN, 1 = TNN, 2 = TBN operands (Ap, Bp as for the corresponding gemm_* call)
 *   out_planes  2: ternary output  y = -1 if c < lo[i], +1 if c > hi[i] (and not c < lo[i]), else 0
 *               1: binary output   y = -1 if c < lo[i], else +1   (hi is not read and may be NULL)
 *   lo, hi      device, int32[M]: thresholds per row i of C (per filter / output channel)
 *   Out         device, N bit strings of depth M in the packed format (string j = column j of C, i.e. one output
 *               pixel; depth position i = output channel): packed_binary_bytes(N, M) or packed_ternary_bytes(N, M)
 *               bytes, overwritten completely (pad bits zero).  This is the layout pack_* produces for an NHWC
 *               feature map with M channels, ready for im2col_packed or as the B operand of the next product.
 */
LB_API int gemm_requant(int kind, int out_planes, int64_t M, int64_t N, int64_t K, const uint64_t *Ap,
                        const uint64_t *Bp, const int32_t *lo, const int32_t *hi, uint64_t *Out, void *stream);

/*
 * Grouped launch: `count` independent products C_p = A_p B_p of one operand class in ONE kernel launch.  The paper's
 * evaluation multiplies many small matrices (Section IV-B: heights 72..360, widths 24..96, depths 128..512), each
 * far too small to occupy this GPU, so a launch per product is bound by launch latency; a group shares one grid.
 *
 *   lb_gemm_problem   the arguments of one gemm_bnn / gemm_tnn / gemm_tbn call (device pointers, same rules).
 *                     Problems with M == 0 or N == 0 are allowed and produce no work.  Output regions of different
 *                     problems must not overlap.
 *   gemm_grouped_table_bytes
 *                     HOST computation: size in bytes of the launch table for these problems, 0 if an argument is
 *                     invalid or the size overflows (lb_last_error() says which).
 *   gemm_grouped_plan HOST computation, no HIP call: validates every problem as gemm_* would and writes the launch
 *                     table into `table` (HOST memory, table_bytes >= gemm_grouped_table_bytes(...)); stores the
 *                     grid size in *workgroups.  The table holds the device pointers and extents of the problems
 *                     and one 32-bit entry per workgroup; it stays valid as long as those pointers do and may be
 *                     reused for any number of launches.
 *   gemm_grouped      enqueues the launch.  table_dev is a DEVICE copy of the planned table (the caller copies it,
 *                     16-byte aligned, and keeps it alive until the work has finished); kind, count and workgroups
 *                     must be the values the table was planned with (the kernel re-checks them against the table
 *                     header and does nothing on a mismatch).  workgroups == 0 is a valid no-op.
 * kind: 0 = BNN, 1 = TNN, 2 = TBN.  Every problem is cut into 16 x 64 output tiles (the small-problem instance of the
 * single-product kernels), so the call suits many small products; one large product is better served by gemm_*.
 */
typedef struct lb_gemm_problem {
    int64_t M, N, K;
    const uint64_t *Ap;
    const uint64_t *Bp;
    int32_t *C;
    int64_t ldc;
} lb_gemm_problem;
LB_API size_t gemm_grouped_table_bytes(int kind, int64_t count, const lb_gemm_problem *problems);
LB_API int gemm_grouped_plan(int kind, int64_t count, const lb_gemm_problem *problems, void *table, size_t table_bytes,
                             int64_t *workgroups);
LB_API int gemm_grouped(int kind, int64_t count, const void *table_dev, int64_t workgroups, void *stream);

/*
 * gemm_grouped_static -- gemm_grouped for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the launch table lives in an array inside the library instead
 * of a device buffer the caller provides.
 *
 *   table_host   HOST memory: the table gemm_grouped_plan wrote for (kind, count, problems); table_bytes its size as
 *                returned by gemm_grouped_table_bytes.  It is read during the call only (its contents travel to the
 *                device inside kernel arguments), so it may be reused or freed as soon as the call returns.
 *   limits       table_bytes <= gemm_grouped_static_max_bytes() (64 KiB: e.g. 512 problems of 16 tiles each);
 *                a larger table is LB_EUNSUPPORTED and nothing is enqueued.  Each GPU the library runs on holds one
 *                such array until the process ends.
 *   The call enqueues ceil(table_bytes / 3584) small upload kernels and the group kernel on `stream`; it calls no
 *   allocating or freeing routine and no memory copy.  Results are those of gemm_grouped on the same table.
 *   Every call on a GPU uses that GPU's one array: calls whose work may overlap on one GPU (different streams, or
 *   several threads without ordering between their streams) race on it and must be serialised by the caller; calls on
 *   one stream are ordered and safe.  The array keeps the last call's table; nothing in it needs clearing, since a call
 *   overwrites every byte its kernel reads.
 * Errors: as gemm_grouped, plus LB_EINVAL when the table does not match kind / count / workgroups.
 */
LB_API size_t gemm_grouped_static_max_bytes(void);
LB_API int gemm_grouped_static(int kind, int64_t count, const void *table_host, size_t table_bytes,
                               int64_t workgroups, void *stream);

/*
 * gemm_i8_mfma -- the same product C = A B from UNPACKED int8 operands with int32 accumulation on the
 * integer matrix cores.  It plays the role the 8-bit gemmlowp multiplication (U8, Section IV, Table II/III)
 * plays in the paper: the comparison point for the low-bit kernels.  Any int8 values are allowed.
 * Right operands of at most 16 columns (with M >= 64) are served by a streaming kernel built on packed 4 x int8 dot
 * products instead of the matrix cores, which such a shape cannot fill.
 *   A  device, int8 row-major M x K, leading dimension lda >= K
 *   B  device, int8 row-major K x N, leading dimension ldb >= N
 *   C  device, int32 row-major M x N, leading dimension ldc >= N; overwritten.
 */
LB_API int gemm_i8_mfma(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                 int32_t *C, int64_t ldc, void *stream);

/*
 * Grouped launch of the 8-bit comparator: `count` independent products C_p = A_p B_p (the arguments of gemm_i8_mfma
 * each) in ONE kernel launch, so that the paper's timing experiment -- many small matrices per algorithm (Section IV-B),
 * ratios between algorithms (Table III) -- compares the packed kernels and the 8-bit comparator launch for launch.
 * Same protocol as gemm_grouped: gemm_i8_grouped_table_bytes and gemm_i8_grouped_plan are HOST computations (the plan
 * validates every problem as gemm_i8_mfma would and writes the launch table into caller-owned host memory);
 * gemm_i8_grouped enqueues the launch on a 16-byte aligned DEVICE copy of that table.  Every problem is cut into
 * 64 x 64 output tiles; operands of any alignment and leading dimension are accepted.  Output regions must not overlap.
 */
typedef struct lb_i8_problem {
    int64_t M, N, K;
    const int8_t *A;
    int64_t lda;
    const int8_t *B;
    int64_t ldb;
    int32_t *C;
    int64_t ldc;
} lb_i8_problem;
LB_API size_t gemm_i8_grouped_table_bytes(int64_t count, const lb_i8_problem *problems);
LB_API int gemm_i8_grouped_plan(int64_t count, const lb_i8_problem *problems, void *table, size_t table_bytes,
                                int64_t *workgroups);
LB_API int gemm_i8_grouped(int64_t count, const void *table_dev, int64_t workgroups, void *stream);

/*
 * gemm_u8_mfma -- 8-bit linear-quantized product with zero points, the scheme of the paper's U8 baseline (eq. (2)
 * and (3), as in gemmlowp):  C[i][j] = sum_t (A[i][t] - zA) * (B[t][j] - zB)  with unsigned 8-bit A, B and integer
 * zero points 0 <= zA, zB <= 255, accumulated in int32.  Computed as eq. (3) prescribes: one matrix product on the
 * matrix cores plus row-sum, column-sum and constant corrections.
 *   A  device, uint8 row-major M x K, lda >= K;  B  device, uint8 row-major K x N, ldb >= N
 *   C  device, int32 row-major M x N, ldc >= N; overwritten.
 *   K <= 33025 so that |C| <= K * 255^2 fits int32 (the paper's eq. (4) bound for unsigned 32-bit is 66051).
 */
LB_API int gemm_u8_mfma(int64_t M, int64_t N, int64_t K, const uint8_t *A, int64_t lda, const uint8_t *B, int64_t ldb,
                        int32_t zA, int32_t zB, int32_t *C, int64_t ldc, void *stream);

/*
 * 4-bit unsigned quantized product with zero points -- the stand-in for the paper's U4 comparison algorithm (Table II,
 * Section IV), computed as eq. (3) prescribes (one matrix product plus row-sum, column-sum and constant corrections):
 *     C[i][j] = sum_t (A[i][t] - zA) * (B[t][j] - zB),   A, B in 0..15,  0 <= zA, zB <= 15,  int32 result.
 * The matrix product runs on the scaled 6-bit floating-point matrix instruction of gfx950 (twice the 8-bit rate): every
 * value v is stored as the 6-bit float v/2 with a block scale of 2, which is exact, and fp32 accumulation of the
 * integer products is exact while 225 * K < 2^24, hence K <= 74565 (LB_EOVERFLOW beyond).
 *
 * Operands are packed beforehand, like the paper's reordered blocks, into the order the multiply reads them:
 *   pack_u4   src   device, one value per byte (only the low 4 bits count); element (r, k) = src[r*stride_r + k*stride_k]
 *                   with stride_k = 1 (A: rows = M, stride_r = lda) or stride_r = 1 (B: rows = N, stride_k = ldb),
 *                   the same rule as pack_binary / pack_ternary
 *             dst   device, 16-byte aligned, packed_u4_bytes(rows, K) bytes: rows padded to multiples of 32 and depth
 *                   to multiples of 128 with zeros; fragment (row block rb, depth block kb of 64) at byte
 *                   (rb * 2*ceil(K/128) + kb) * 1536; inside it three planes of 64 slots x 8 bytes, slot 32*h + i =
 *                   depth positions 64*kb + 32*h .. + 31 of row 32*rb + i as a 192-bit little-endian string (position j
 *                   in bits 6j .. 6j+5, plane p = bits 64p .. 64p+63)
 *             sums  device, int32[rows]: sum of the K values of each row (overwritten)
 *             Enqueues two kernels on `stream`.  rows == 0 or K == 0: nothing is written.
 *   gemm_u4_mfma    Ap / sumA from pack_u4 of A (M strings), Bp / sumB from pack_u4 of B (N strings), same K;
 *                   C device, int32 row-major M x N, ldc >= N, overwritten.  May enqueue two kernels (column ranges
 *                   of C with different tile sizes).
 * Errors as for the other entry points (LB_EINVAL for null / misaligned pointers, bad strides, zero points outside
 * 0..15, K < 1; LB_EOVERFLOW for K > 74565, for rows beyond 2^31 - 1 in pack_u4 and for M or N beyond 2^31 - 256 in
 * gemm_u4_mfma).
 */
LB_API size_t packed_u4_bytes(int64_t rows, int64_t K);
LB_API int pack_u4(const uint8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, void *dst,
                   int32_t *sums, void *stream);
LB_API int gemm_u4_mfma(int64_t M, int64_t N, int64_t K, const void *Ap, const int32_t *sumA, const void *Bp,
                        const int32_t *sumB, int32_t zA, int32_t zB, int32_t *C, int64_t ldc, void *stream);

/*
 * The paper's product C = A B over {-1, 0, +1} (Section II-A; value sets of Section III-A: any mix of ternary and
 * binary operands) on the matrix cores instead of AND / XOR / popcount: both operands stored as 4-bit floats (1 sign,
 * 2 exponent, 1 mantissa bit, bias 1; 0 and +-1 are exact), multiplied by the scaled low-precision matrix instruction of
 * gfx950 with fp32 accumulation, which is exact while |C| <= K < 2^24 (LB_EOVERFLOW beyond).  Not the paper's algorithm:
 * the point of comparison for it on hardware that has 4-bit matrix arithmetic.  4 bits per value instead of 2 or 1.
 *   pack_t4       src   device, int8, taken by sign like pack_ternary (x > 0 -> +1, x < 0 -> -1); element (r, k) =
 *                       src[r*stride_r + k*stride_k] with stride_k = 1 or stride_r = 1 (same rule as pack_ternary)
 *                 dst   device, 16-byte aligned, packed_t4_bytes(rows, K) bytes: rows padded to multiples of 32, depth
 *                       to multiples of 128 with zeros; fragment (row block rb, depth block kb of 64) at byte
 *                       (rb * 2*ceil(K/128) + kb) * 1024; inside it 64 slots of 16 bytes, slot 32*h + i = depth positions
 *                       64*kb + 32*h .. + 31 of row 32*rb + i, position j in bits 4j .. 4j+3 (little-endian)
 *   gemm_t4_mfma  Ap from pack_t4 of A (M strings), Bp from pack_t4 of B (N strings), same K; C device, int32
 *                 row-major M x N, ldc >= N, overwritten.  May enqueue two kernels (column ranges of C with different
 *                 tile sizes).
 * Errors as for the other entry points; LB_EOVERFLOW for K >= 2^24 and for M or N beyond 2^31 - 256.
 */
LB_API size_t packed_t4_bytes(int64_t rows, int64_t K);
LB_API int pack_t4(const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, void *dst,
                   void *stream);
LB_API int gemm_t4_mfma(int64_t M, int64_t N, int64_t K, const void *Ap, const void *Bp, int32_t *C, int64_t ldc,
                        void *stream);

/*
 * Which kernel a gemm_bnn / gemm_tnn / gemm_tbn call (c16 = 0) or a gemm_c16 call (c16 = 1) of this shape would run:
 * host logic only, usable without a GPU.  kind 0 = BNN, 1 = TNN, 2 = TBN.  Returns a short description (thread-local
 * host string, valid until the next call on the thread), or NULL for arguments the gemm calls would reject.
 */
LB_API const char *lb_describe_plan(int kind, int64_t M, int64_t N, int64_t K, int c16);

#ifdef __cplusplus
}
#endif
#endif /* LOWBIT_GEMM_H */
