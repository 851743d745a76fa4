// C ABI of the library: argument validation, shape-based kernel selection, error reporting.
// Every check runs before the first HIP call, so invalid requests can be rejected on a machine without a GPU.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>

#include "../../include/lowbit_gemm.h"
#include "../../include/lowbit_gemm_bench.h"
#include "lowbit_internal.h"

namespace {

thread_local char g_err[256] = "";
// benchmark hook (lb_set_variant): forced tile variant per gemm entry point; every call reads its slot once
std::atomic<int> g_forced[3] = {{-1}, {-1}, {-1}};
int forced_variant(int kind) { return g_forced[kind].load(std::memory_order_relaxed); }

int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// The library holds machine code for gfx950 only.  Every entry point asks this before its first launch on a device
// (the answer is cached per device), so that a call on another GPU fails with a clear status instead of a launch error.
bool arch_supported(const char *arch)
{
    // "gfx950" alone or followed by feature flags ("gfx950:sramecc+:xnack-")
    return arch && strncmp(arch, "gfx950", 6) == 0 && (arch[6] == '\0' || arch[6] == ':');
}

constexpr int kMaxDevices = 64;
std::atomic<signed char> g_arch_state[kMaxDevices];  // 0 = not asked yet, 1 = gfx950, -1 = something else

int check_device(const char *name)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(LB_EUNSUPPORTED, "%s: device index %d beyond %d", name, dev, kMaxDevices - 1);
    signed char st = g_arch_state[dev].load(std::memory_order_relaxed);
    if (st == 0) {
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, dev);
        if (e != hipSuccess)
            return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
        st = arch_supported(prop.gcnArchName) ? 1 : -1;
        g_arch_state[dev].store(st, std::memory_order_relaxed);
        if (st < 0)
            return fail(LB_EUNSUPPORTED, "%s: device %d is %s; this library is built for gfx950 only", name, dev,
                        prop.gcnArchName);
    }
    if (st < 0)
        return fail(LB_EUNSUPPORTED, "%s: device %d is not gfx950; this library is built for gfx950 only", name, dev);
    return LB_OK;
}

constexpr int64_t kMaxDepth = 0x7fffffffLL;    // int32 accumulators: |c| <= K must fit
constexpr int64_t kMaxExtent = 0x7fffffffLL;   // kernels index bit strings with 32-bit integers

constexpr int64_t kU4MaxDepth = 74565;         // 225 * K < 2^24: fp32 sums of 4-bit products stay exact
constexpr int64_t kMxMaxExtent = 0x7fffff00LL;  // matrix-core kernels: row / column indices of a 256-wide tile stay in int32
constexpr int64_t kT4MaxDepth = 16777215;      // K < 2^24: fp32 sums of +-1 products stay exact
constexpr int64_t kSkinnyMax = 32;             // widest "skinny" side served by the depth-split kernel
constexpr int kI8Instances = 10;               // kernel instances of gemm_i8_mfma selectable through lb_set_variant

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// rows*ceil(K/64)*unit with overflow detection; 0 on failure
size_t packed_bytes(int64_t rows, int64_t K, int64_t unit)
{
    if (rows < 0 || K < 0)
        return 0;
    const int64_t KW = K / 64 + (K % 64 != 0);
    if (rows == 0 || KW == 0)
        return 0;
    if (KW > INT64_MAX / unit || rows > INT64_MAX / (KW * unit))
        return 0;
    return (size_t)(rows * KW * unit);
}

// Argument rules shared by every packing entry point.  *nothing is set when rows == 0 or K == 0 (valid, nothing to do);
// *k_contig tells which of the two accepted source layouts was given.
int check_pack(const char *name, const void *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k,
               const void *dst, int64_t max_depth, bool *nothing, bool *k_contig)
{
    *nothing = false;
    if (rows < 0 || K < 0)
        return fail(LB_EINVAL, "%s: rows=%lld K=%lld must be >= 0", name, (long long)rows, (long long)K);
    if (rows == 0 || K == 0) {
        *nothing = true;
        return LB_OK;
    }
    if (!src || !dst)
        return fail(LB_EINVAL, "%s: null pointer", name);
    if (K > max_depth || rows > kMaxExtent)
        return fail(LB_EOVERFLOW, "%s: rows=%lld K=%lld exceed 2^31-1 rows / %lld depth positions", name,
                    (long long)rows, (long long)K, (long long)max_depth);
    // a single bit string (rows == 1) or a single depth position (K == 1) makes the other stride irrelevant
    *k_contig = stride_k == 1 && (rows == 1 || stride_r >= K);
    const bool k_strided = stride_r == 1 && (K == 1 || stride_k >= rows);
    if (stride_r < 1 || stride_k < 1 || !(*k_contig || k_strided))
        return fail(LB_EINVAL,
                    "%s: need stride_k=1 with stride_r>=K, or stride_r=1 with stride_k>=rows (got stride_r=%lld "
                    "stride_k=%lld rows=%lld K=%lld)",
                    name, (long long)stride_r, (long long)stride_k, (long long)rows, (long long)K);
    if (stride_r > INT64_MAX / rows || stride_k > INT64_MAX / K)
        return fail(LB_EOVERFLOW, "%s: source extent overflows", name);
    if (!aligned(dst, 16))
        return fail(LB_EINVAL, "%s: dst must be 16-byte aligned", name);
    return LB_OK;
}

int do_pack(bool ternary, const char *name, const int8_t *src, int64_t rows, int64_t K, int64_t stride_r,
            int64_t stride_k, uint64_t *dst, void *stream)
{
    bool nothing, k_contig;
    const int rc = check_pack(name, src, rows, K, stride_r, stride_k, dst, kMaxDepth, &nothing, &k_contig);
    if (rc != LB_OK || nothing)
        return rc;
    if (packed_bytes(rows, K, ternary ? 16 : 8) == 0)
        return fail(LB_EOVERFLOW, "%s: packed size overflows", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e =
        lowbit::launch_pack(ternary, src, rows, K, stride_r, stride_k, dst, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

// Pick a tile variant.  Problems of a few hundred 16 x 64 tiles are latency-bound and take the first matching
// small-problem instance of the table; otherwise the highest-ranked variant that still yields enough workgroups
// (six per compute unit for the 32 x 64 tile of rank 2, eight for the larger tiles), and failing that the ranked
// variant with the most workgroups.  A scalar side of at most 8 (16) strings only admits tiles of at most 8 (16)
// rows, so that no wave multiplies padding.
// base_only: leave out the instances that ask for a minimum depth (eight waves of four rows on a 32 x 128 or 32 x 64
// tile), which were tuned on plain products.  conv_gemm: a thread pays the gather's bounds check and address once per stage, and those
// instances stage half as many words per thread (headline layer: 745 us with the 32 x 256 tile of four waves, 787 us
// with them).  gemm_requant: 755 against 774 us on the same layer.
int choose_variant(const lowbit::GemmVariant *tab, int count, int64_t rowsS, int64_t rowsV, int64_t KW,
                   bool base_only = false)
{
    const int max_tile_s = rowsS <= 8 ? 8 : rowsS <= 16 ? 16 : 1 << 30;
    const int64_t n16 = ((rowsS + 15) / 16) * ((rowsV + 63) / 64);
    for (int i = 0; i < count; ++i)
        if (tab[i].small_max > 0 && tab[i].tileS <= max_tile_s && n16 <= tab[i].small_max && KW >= tab[i].small_min_kw)
            return i;
    int best = -1, fallback = -1;
    int64_t fallback_wg = -1;
    for (int i = 0; i < count; ++i) {
        if (tab[i].rank <= 0 || tab[i].tileS > max_tile_s || KW < tab[i].small_min_kw ||
            (base_only && tab[i].wanted_wg > 0 && tab[i].small_min_kw > 0))
            continue;
        const int64_t wg = ((rowsS + tab[i].tileS - 1) / tab[i].tileS) * ((rowsV + tab[i].tileV - 1) / tab[i].tileV);
        const int64_t wanted = tab[i].wanted_wg > 0 ? tab[i].wanted_wg : tab[i].rank <= 2 ? 256 * 6 : 256 * 8;
        // an instance with a threshold of its own is also taken when its workgroups fill whole rounds of two per
        // compute unit (512 x 4096 x 2304: 512 tiles of 32 x 128, 14 % faster; 576 tiles: 6 % slower)
        const bool fills = tab[i].wanted_wg > 0 && wg >= 512 && wg % 256 == 0;
        if ((wg >= wanted || fills) && (best < 0 || tab[i].rank > tab[best].rank))
            best = i;
        if (wg > fallback_wg) {
            fallback_wg = wg;
            fallback = i;
        }
    }
    if (best >= 0)
        return best;
    if (fallback >= 0)
        return fallback;
    // no ranked variant is low enough: the tallest 64-column instance that is
    int fit = 0;
    bool found = false;
    for (int i = 0; i < count; ++i)
        if (tab[i].tileV == 64 && tab[i].tileS <= max_tile_s && (!found || tab[i].tileS > tab[fit].tileS)) {
            fit = i;
            found = true;
        }
    return fit;
}

// Argument rules common to gemm_bnn / gemm_tnn / gemm_tbn and to every problem of a grouped launch.
// *empty is set when there is nothing to compute (M == 0 or N == 0).
int check_gemm(const char *name, int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp,
               const void *C, int64_t ldc, bool *empty, int c_bytes = 4)
{
    *empty = false;
    if (M < 0 || N < 0)
        return fail(LB_EINVAL, "%s: M=%lld N=%lld must be >= 0", name, (long long)M, (long long)N);
    if (K <= 0)
        return fail(LB_EINVAL, "%s: K=%lld must be >= 1", name, (long long)K);
    if (K > kMaxDepth)
        return fail(LB_EOVERFLOW, "%s: K=%lld exceeds 2^31-1 (int32 accumulators)", name, (long long)K);
    if (M > kMaxExtent || N > kMaxExtent)
        return fail(LB_EOVERFLOW, "%s: M=%lld N=%lld exceed 2^31-1", name, (long long)M, (long long)N);
    if (M == 0 || N == 0) {
        *empty = true;
        return LB_OK;
    }
    if (!Ap || !Bp || !C)
        return fail(LB_EINVAL, "%s: null pointer", name);
    if (ldc < N)
        return fail(LB_EINVAL, "%s: ldc=%lld < N=%lld", name, (long long)ldc, (long long)N);
    if (ldc > INT64_MAX / M / c_bytes)
        return fail(LB_EOVERFLOW, "%s: M*ldc overflows", name);
    if (!aligned(Ap, 16) || !aligned(Bp, 16) || !aligned(C, (uintptr_t)c_bytes))
        return fail(LB_EINVAL, "%s: operands must be 16-byte aligned, C %d-byte aligned", name, c_bytes);
    return LB_OK;
}

// Depth-split (skinny) kernel or tiled kernel for a product with at most 32 strings on one side?  The skinny kernel
// streams the `rows` long strings once (8, 16 or 32 short strings per workgroup) and pays a cross-lane reduction per
// row, so it wins when the depth is large against the row count; the tiled kernel wins on many shallow rows (measured
// over rows 1 K .. 256 K, depth 1 K .. 64 K, 1 .. 32 short strings: up to 10x either way).
bool prefer_skinny(int64_t rows, int64_t narrow, int64_t K)
{
    if (lowbit::skinny_forced_config() >= 0)  // a forced configuration of that kernel also forces the kernel
        return true;
    if (K < 2048)
        return false;
    if (narrow <= 8)
        return K >= 16384 || rows <= K;
    if (K < 4096)
        return false;
    if (narrow <= 16)
        return rows <= (K < 16384 ? K : 16384);
    return rows <= (K / 4 < 8192 ? K / 4 : 8192);
}

// Which operand rides in scalar registers.  TBN: always the binary one (one scalar source per instruction), so lanes
// own rows of C.  BNN / TNN: lanes own columns of C (coalesced stores) unless N is too narrow to fill a wavefront and
// M is not.
bool b_on_scalar_side(int kind, int64_t M, int64_t N) { return kind == lowbit::KIND_TBN || (N < 64 && M > N); }

// How one gemm_bnn / gemm_tnn / gemm_tbn / gemm_c16 call is carried out: host logic only, no HIP call.
struct GemmPlan {
    enum Path { SKINNY, SPLIT, TILED } path;
    int kind;         // launcher kind (KIND_TBN_SV when gemm_tbn swaps the operand roles)
    bool transposed;  // tiled / split: B on the scalar side, lanes own rows of C; skinny: B is the streamed operand
    int variant;      // tiled: index into gemm_variants(kind)
    int nsplit;       // split: depth ranges
};

GemmPlan plan_gemm(int kind, int64_t M, int64_t N, int64_t K, bool c16)
{
    GemmPlan p{GemmPlan::TILED, kind, false, 0, 1};
    const int64_t KW = (K + 63) / 64;
    int count = 0;
    const lowbit::GemmVariant *tab = lowbit::gemm_variants(kind, &count);
    const int fv = forced_variant(kind);
    const bool forced = fv >= 0 && fv < count;

    // Skinny problems (fully connected layers with a small batch) stream the large operand once and split the
    // depth across lanes.  A forced tile variant bypasses this path.
    if (!forced) {
        const bool narrow_n = N <= kSkinnyMax && M >= 64;
        const bool narrow_m = !narrow_n && M <= kSkinnyMax && N >= 64;
        const bool skinny_n = narrow_n && prefer_skinny(M, N, K);
        const bool skinny_m = narrow_m && prefer_skinny(N, M, K);
        if (skinny_n || skinny_m) {
            p.path = GemmPlan::SKINNY;
            p.transposed = skinny_m;
            // gemm_tbn with few ternary rows: the binary operand is the streamed one
            if (kind == lowbit::KIND_TBN && skinny_m)
                p.kind = lowbit::KIND_TBN_SV;
            return p;
        }
    }
    // gemm_tbn normally keeps the binary operand on the scalar side (2 instructions per word, lanes own rows of C).
    // With at most 32 ternary rows most of those lanes would idle: then the ternary operand goes to the scalar side
    // (3 instructions per word, lanes own columns of C).
    if (kind == lowbit::KIND_TBN && !forced && M <= 32 && N > M) {
        p.kind = lowbit::KIND_TBN_SV;
        tab = lowbit::gemm_variants(p.kind, &count);
    }
    p.transposed = p.kind != lowbit::KIND_TBN_SV && b_on_scalar_side(p.kind, M, N);
    const int64_t rowsS = p.transposed ? N : M, rowsV = p.transposed ? M : N;
    // Few tiles and a long depth: every workgroup would walk the whole depth, one dependent memory round trip after
    // the other, on a mostly idle machine.  Split the depth over enough workgroups to give each compute unit about
    // six (at least 16 depth words per split); the partial products are added into a cleared C (measured: 128 x 128 x
    // 16384 3x faster, 64 x 64 x 65536 11x, 512 x 49 x 65536 3x; below these depths the cleared C and the atomic adds
    // cost more than the split gains).
    const int64_t split_min_kw = kind == lowbit::KIND_TNN ? 128 : 160;
    if (!forced && !c16 && KW >= split_min_kw && M <= 65535) {
        const int64_t tiles8 = ((rowsS + 7) / 8) * ((rowsV + 63) / 64);
        int64_t nsplit = 1536 / tiles8;
        if (nsplit > KW / 16)
            nsplit = KW / 16;
        if (tiles8 <= 208 && nsplit >= 2) {
            p.path = GemmPlan::SPLIT;
            p.nsplit = (int)nsplit;
            return p;
        }
    }
    p.variant = forced ? fv : choose_variant(tab, count, rowsS, rowsV, KW);
    return p;
}

// c16: C is an int16_t matrix (passed as void through the int32_t pointer of the launch arguments).
int do_gemm(int kind, const char *name, int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp,
            void *C, int64_t ldc, void *stream, bool c16 = false)
{
    bool empty;
    const int rc = check_gemm(name, M, N, K, Ap, Bp, C, ldc, &empty, c16 ? 2 : 4);
    if (rc != LB_OK || empty)
        return rc;
    const int64_t KW = (K + 63) / 64;
    const GemmPlan p = plan_gemm(kind, M, N, K, c16);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    hipError_t e;
    if (p.path == GemmPlan::SKINNY) {
        const bool b_streamed = p.transposed;
        lowbit::SkinnyArgs sa;
        sa.Xp = b_streamed ? Bp : Ap;
        sa.Yp = b_streamed ? Ap : Bp;
        sa.rowsX = (int)(b_streamed ? N : M);
        sa.rowsY = (int)(b_streamed ? M : N);
        sa.KW = (int)KW;
        sa.K = (int)K;
        sa.C = static_cast<int32_t *>(C);
        sa.ldc = ldc;
        sa.c16 = c16 ? 1 : 0;
        sa.stream = static_cast<hipStream_t>(stream);
        e = lowbit::launch_gemm_skinny(p.kind, sa, b_streamed);
    } else {
        lowbit::GemmArgs a;
        a.Sp = reinterpret_cast<const uint32_t *>(p.transposed ? Bp : Ap);
        a.rowsS = (int)(p.transposed ? N : M);
        a.Vp = reinterpret_cast<const uint32_t *>(p.transposed ? Ap : Bp);
        a.rowsV = (int)(p.transposed ? M : N);
        a.KW = (int)KW;
        a.K = (int)K;
        a.C = static_cast<int32_t *>(C);
        a.ldc = ldc;
        a.c16 = c16 ? 1 : 0;
        a.stream = static_cast<hipStream_t>(stream);
        if (p.path == GemmPlan::SPLIT) {
            e = lowbit::launch_gemm_splitk(p.kind, a, p.transposed, p.nsplit);
        } else {
            int count = 0;
            const lowbit::GemmVariant *tab = lowbit::gemm_variants(p.kind, &count);
            e = p.transposed ? tab[p.variant].launch_transposed(a) : tab[p.variant].launch(a);
        }
    }
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

// Validates every problem of a group and counts the workgroups the launch needs.
int group_workgroups(int kind, const char *name, int64_t count, const lb_gemm_problem *problems, int64_t *workgroups)
{
    if (kind < 0 || kind > 2)
        return fail(LB_EINVAL, "%s: kind=%d must be 0 (BNN), 1 (TNN) or 2 (TBN)", name, kind);
    if (count < 0 || (count > 0 && !problems))
        return fail(LB_EINVAL, "%s: count=%lld with problems=%p", name, (long long)count, (const void *)problems);
    if (count > 0x7fffffffLL)
        return fail(LB_EOVERFLOW, "%s: count=%lld exceeds 2^31-1", name, (long long)count);
    int64_t total = 0;
    for (int64_t p = 0; p < count; ++p) {
        const lb_gemm_problem &q = problems[p];
        bool empty;
        char where[48];
        snprintf(where, sizeof(where), "%s: problem %lld", name, (long long)p);
        const int rc = check_gemm(where, q.M, q.N, q.K, q.Ap, q.Bp, q.C, q.ldc, &empty);
        if (rc != LB_OK)
            return rc;
        if (empty)
            continue;
        const bool tr = b_on_scalar_side(kind, q.M, q.N);
        const int64_t rowsS = tr ? q.N : q.M, rowsV = tr ? q.M : q.N;
        total += ((rowsS + lowbit::kGroupTileS - 1) / lowbit::kGroupTileS) *
                 ((rowsV + lowbit::kGroupTileV - 1) / lowbit::kGroupTileV);
        if (total > 0x7fffffffLL)
            return fail(LB_EOVERFLOW, "%s: more than 2^31-1 workgroups", name);
    }
    *workgroups = total;
    return LB_OK;
}

// Argument rules of gemm_i8_mfma, also applied to every problem of its grouped launch.
int check_gemm_i8(const char *name, int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B,
                  int64_t ldb, const int32_t *C, int64_t ldc, bool *empty)
{
    *empty = false;
    if (M < 0 || N < 0)
        return fail(LB_EINVAL, "%s: M=%lld N=%lld must be >= 0", name, (long long)M, (long long)N);
    if (K <= 0)
        return fail(LB_EINVAL, "%s: K=%lld must be >= 1", name, (long long)K);
    // |a*b| <= 2^14, so the int32 sum is safe up to K = 2^17 - 1 for arbitrary int8 inputs
    if (K > 131071)
        return fail(LB_EOVERFLOW, "%s: K=%lld exceeds 131071 (int32 accumulation of int8 products)", name,
                    (long long)K);
    if (M > kMaxExtent || N > kMaxExtent)
        return fail(LB_EOVERFLOW, "%s: M=%lld N=%lld exceed 2^31-1", name, (long long)M, (long long)N);
    if (M == 0 || N == 0) {
        *empty = true;
        return LB_OK;
    }
    if (!A || !B || !C)
        return fail(LB_EINVAL, "%s: null pointer", name);
    if (lda < K || ldb < N || ldc < N)
        return fail(LB_EINVAL, "%s: lda=%lld ldb=%lld ldc=%lld too small", name, (long long)lda, (long long)ldb,
                    (long long)ldc);
    if (lda > INT64_MAX / M || ldb > INT64_MAX / K || ldc > INT64_MAX / M / 4)
        return fail(LB_EOVERFLOW, "%s: matrix extent overflows", name);
    if (!aligned(C, 4))
        return fail(LB_EINVAL, "%s: C must be 4-byte aligned", name);
    return LB_OK;
}

int i8_group_workgroups(const char *name, int64_t count, const lb_i8_problem *problems, int64_t *workgroups)
{
    if (count < 0 || (count > 0 && !problems))
        return fail(LB_EINVAL, "%s: count=%lld with problems=%p", name, (long long)count, (const void *)problems);
    if (count > 0x7fffffffLL)
        return fail(LB_EOVERFLOW, "%s: count=%lld exceeds 2^31-1", name, (long long)count);
    int64_t total = 0;
    constexpr int T = lowbit::kI8GroupTile;
    for (int64_t p = 0; p < count; ++p) {
        const lb_i8_problem &q = problems[p];
        bool empty;
        char where[48];
        snprintf(where, sizeof(where), "%s: problem %lld", name, (long long)p);
        const int rc = check_gemm_i8(where, q.M, q.N, q.K, q.A, q.lda, q.B, q.ldb, q.C, q.ldc, &empty);
        if (rc != LB_OK)
            return rc;
        if (empty)
            continue;
        total += ((q.M + T - 1) / T) * ((q.N + T - 1) / T);
        if (total > 0x7fffffffLL)
            return fail(LB_EOVERFLOW, "%s: more than 2^31-1 workgroups", name);
    }
    *workgroups = total;
    return LB_OK;
}

size_t i8_group_table_bytes(int64_t count, int64_t workgroups)
{
    const size_t raw = sizeof(lowbit::I8GroupHeader) + (size_t)count * sizeof(lowbit::I8GroupRecord) +
                       (size_t)workgroups * sizeof(uint32_t);
    return (raw + 15) & ~(size_t)15;
}

// Geometry rules shared by im2col_packed and conv_gemm; fills *g.  *empty: nothing to compute (batch == 0 or a window
// larger than the padded map).
int check_conv_geom(const char *name, int64_t batch, int64_t H, int64_t W, int64_t C, int kh, int kw, int stride_h,
                    int stride_w, int pad_h, int pad_w, lowbit::Im2colGeom *g, bool *empty)
{
    *empty = false;
    if (batch < 0 || H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 ||
        pad_w < 0)
        return fail(LB_EINVAL, "%s: bad geometry batch=%lld H=%lld W=%lld C=%lld window %dx%d stride %dx%d pad %dx%d",
                    name, (long long)batch, (long long)H, (long long)W, (long long)C, kh, kw, stride_h, stride_w, pad_h,
                    pad_w);
    if (C % 64 != 0)
        return fail(LB_EUNSUPPORTED, "%s: C=%lld is not a multiple of 64", name, (long long)C);
    constexpr int64_t kLim = 1 << 24;  // keeps every product below in 64 bits and the map extents in 32
    if (H > kLim || W > kLim || C > kLim * 64 || kh > 4096 || kw > 4096 || stride_h > kLim || stride_w > kLim ||
        pad_h > kLim || pad_w > kLim || batch > kMaxExtent)
        return fail(LB_EOVERFLOW, "%s: geometry too large", name);
    const int64_t OH = (H + 2 * pad_h - kh) >= 0 ? (H + 2 * pad_h - kh) / stride_h + 1 : 0;
    const int64_t OW = (W + 2 * pad_w - kw) >= 0 ? (W + 2 * pad_w - kw) / stride_w + 1 : 0;
    if (batch == 0 || OH == 0 || OW == 0) {
        *empty = true;
        return LB_OK;
    }
    const int64_t CW = C / 64;
    const int64_t kwout = (int64_t)kh * kw * CW;
    if (kwout > kMaxExtent / 64 || OH * OW > kMaxExtent || batch > INT64_MAX / (OH * OW) / kwout / 16)
        return fail(LB_EOVERFLOW, "%s: packed operand too large", name);
    g->batch = batch;
    g->H = (int)H;
    g->W = (int)W;
    g->CW = (int)CW;
    g->OH = (int)OH;
    g->OW = (int)OW;
    g->kh = kh;
    g->kw = kw;
    g->sh = stride_h;
    g->sw = stride_w;
    g->ph = pad_h;
    g->pw = pad_w;
    return LB_OK;
}

size_t group_table_bytes(int64_t count, int64_t workgroups)
{
    // header + records + one entry per workgroup, rounded up to 16 bytes
    const size_t raw = sizeof(lowbit::GroupHeader) + (size_t)count * sizeof(lowbit::GroupRecord) +
                       (size_t)workgroups * sizeof(uint32_t);
    return (raw + 15) & ~(size_t)15;
}

}  // namespace

extern "C" {

const char *lb_last_error(void) { return g_err; }

int lb_format_version(void) { return LB_FORMAT_VERSION; }

int lb_arch_supported(const char *gcn_arch_name) { return arch_supported(gcn_arch_name) ? 1 : 0; }

size_t packed_binary_bytes(int64_t rows, int64_t K) { return packed_bytes(rows, K, 8); }

size_t packed_ternary_bytes(int64_t rows, int64_t K) { return packed_bytes(rows, K, 16); }

int pack_binary(const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, uint64_t *dst,
                void *stream)
{
    return do_pack(false, "pack_binary", src, rows, K, stride_r, stride_k, dst, stream);
}

int pack_ternary(const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, uint64_t *dst,
                 void *stream)
{
    return do_pack(true, "pack_ternary", src, rows, K, stride_r, stride_k, dst, stream);
}

int gemm_bnn(int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp, int32_t *C, int64_t ldc,
             void *stream)
{
    return do_gemm(lowbit::KIND_BNN, "gemm_bnn", M, N, K, Ap, Bp, C, ldc, stream);
}

int gemm_tnn(int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp, int32_t *C, int64_t ldc,
             void *stream)
{
    return do_gemm(lowbit::KIND_TNN, "gemm_tnn", M, N, K, Ap, Bp, C, ldc, stream);
}

int gemm_tbn(int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp, int32_t *C, int64_t ldc,
             void *stream)
{
    return do_gemm(lowbit::KIND_TBN, "gemm_tbn", M, N, K, Ap, Bp, C, ldc, stream);
}

int gemm_c16(int kind, int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp, int16_t *C, int64_t ldc,
             void *stream)
{
    const char *name = "gemm_c16";
    if (kind < 0 || kind > 2)
        return fail(LB_EINVAL, "%s: kind=%d must be 0 (BNN), 1 (TNN) or 2 (TBN)", name, kind);
    // |c| <= K for every kind, so a signed 16-bit C is exact up to the k_max of Table II
    if (K > 32767)
        return fail(LB_EOVERFLOW, "%s: K=%lld exceeds 32767 (signed 16-bit C)", name, (long long)K);
    return do_gemm(kind, name, M, N, K, Ap, Bp, C, ldc, stream, true);
}

size_t gemm_grouped_table_bytes(int kind, int64_t count, const lb_gemm_problem *problems)
{
    int64_t wg = 0;
    if (group_workgroups(kind, "gemm_grouped_table_bytes", count, problems, &wg) != LB_OK)
        return 0;
    return group_table_bytes(count, wg);
}

int gemm_grouped_plan(int kind, int64_t count, const lb_gemm_problem *problems, void *table, size_t table_bytes,
                      int64_t *workgroups)
{
    const char *name = "gemm_grouped_plan";
    if (!table || !workgroups)
        return fail(LB_EINVAL, "%s: null pointer", name);
    int64_t wg = 0;
    const int rc = group_workgroups(kind, name, count, problems, &wg);
    if (rc != LB_OK)
        return rc;
    const size_t need = group_table_bytes(count, wg);
    if (table_bytes < need)
        return fail(LB_EINVAL, "%s: table_bytes=%zu < %zu", name, table_bytes, need);
    memset(table, 0, need);
    auto *hdr = static_cast<lowbit::GroupHeader *>(table);
    auto *recs = reinterpret_cast<lowbit::GroupRecord *>(hdr + 1);
    auto *owner = reinterpret_cast<uint32_t *>(recs + count);
    hdr->magic = lowbit::kGroupMagic;
    hdr->kind = (uint32_t)kind;
    hdr->count = (uint32_t)count;
    hdr->workgroups = (uint32_t)wg;
    uint32_t next = 0;
    for (int64_t p = 0; p < count; ++p) {
        const lb_gemm_problem &q = problems[p];
        lowbit::GroupRecord &r = recs[p];
        r.tile0 = next;
        if (q.M == 0 || q.N == 0)
            continue;  // owns no workgroup; the zeroed record is never read
        const bool tr = b_on_scalar_side(kind, q.M, q.N);
        r.Sp = reinterpret_cast<const uint32_t *>(tr ? q.Bp : q.Ap);
        r.Vp = reinterpret_cast<const uint32_t *>(tr ? q.Ap : q.Bp);
        r.C = q.C;
        r.ldc = q.ldc;
        r.rowsS = (int32_t)(tr ? q.N : q.M);
        r.rowsV = (int32_t)(tr ? q.M : q.N);
        r.KW = (int32_t)((q.K + 63) / 64);
        r.K = (int32_t)q.K;
        r.nSB = (r.rowsS + lowbit::kGroupTileS - 1) / lowbit::kGroupTileS;
        r.transposed = tr ? 1 : 0;
        const uint32_t tiles = (uint32_t)r.nSB * (uint32_t)((r.rowsV + lowbit::kGroupTileV - 1) / lowbit::kGroupTileV);
        for (uint32_t t = 0; t < tiles; ++t)
            owner[next + t] = (uint32_t)p;
        next += tiles;
    }
    *workgroups = wg;
    return LB_OK;
}

int gemm_grouped(int kind, int64_t count, const void *table_dev, int64_t workgroups, void *stream)
{
    const char *name = "gemm_grouped";
    if (kind < 0 || kind > 2)
        return fail(LB_EINVAL, "%s: kind=%d must be 0 (BNN), 1 (TNN) or 2 (TBN)", name, kind);
    if (count < 0 || workgroups < 0)
        return fail(LB_EINVAL, "%s: count=%lld workgroups=%lld must be >= 0", name, (long long)count,
                    (long long)workgroups);
    if (count > 0x7fffffffLL || workgroups > 0x7fffffffLL)
        return fail(LB_EOVERFLOW, "%s: count=%lld workgroups=%lld exceed 2^31-1", name, (long long)count,
                    (long long)workgroups);
    if (workgroups == 0)
        return LB_OK;
    if (count == 0)
        return fail(LB_EINVAL, "%s: %lld workgroups for no problems", name, (long long)workgroups);
    if (!table_dev || !aligned(table_dev, 16))
        return fail(LB_EINVAL, "%s: table_dev must be a 16-byte aligned device pointer", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e =
        lowbit::launch_gemm_group(kind, static_cast<const lowbit::GroupHeader *>(table_dev), (uint32_t)count,
                                  (uint32_t)workgroups, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

size_t gemm_grouped_static_max_bytes(void) { return lowbit::kGroupStaticBytes; }

int gemm_grouped_static(int kind, int64_t count, const void *table_host, size_t table_bytes, int64_t workgroups,
                        void *stream)
{
    const char *name = "gemm_grouped_static";
    if (kind < 0 || kind > 2)
        return fail(LB_EINVAL, "%s: kind=%d must be 0 (BNN), 1 (TNN) or 2 (TBN)", name, kind);
    if (count < 0 || workgroups < 0)
        return fail(LB_EINVAL, "%s: count=%lld workgroups=%lld must be >= 0", name, (long long)count,
                    (long long)workgroups);
    if (count > 0x7fffffffLL || workgroups > 0x7fffffffLL)
        return fail(LB_EOVERFLOW, "%s: count=%lld workgroups=%lld exceed 2^31-1", name, (long long)count,
                    (long long)workgroups);
    if (workgroups == 0)
        return LB_OK;
    if (count == 0)
        return fail(LB_EINVAL, "%s: %lld workgroups for no problems", name, (long long)workgroups);
    if (!table_host)
        return fail(LB_EINVAL, "%s: table_host is null", name);
    // the table must be the one gemm_grouped_plan wrote for these values: its size follows from them
    const size_t need = group_table_bytes(count, workgroups);
    if (table_bytes != need)
        return fail(LB_EINVAL, "%s: table_bytes=%zu, but a table of %lld problems and %lld workgroups has %zu", name,
                    table_bytes, (long long)count, (long long)workgroups, need);
    if (table_bytes > lowbit::kGroupStaticBytes)
        return fail(LB_EUNSUPPORTED, "%s: table of %zu bytes exceeds the library's %zu-byte array (use gemm_grouped)",
                    name, table_bytes, (size_t)lowbit::kGroupStaticBytes);
    const auto *hdr = static_cast<const lowbit::GroupHeader *>(table_host);
    if (hdr->magic != lowbit::kGroupMagic || hdr->kind != (uint32_t)kind || hdr->count != (uint32_t)count ||
        hdr->workgroups != (uint32_t)workgroups)
        return fail(LB_EINVAL, "%s: the table was not planned for kind=%d count=%lld workgroups=%lld", name, kind,
                    (long long)count, (long long)workgroups);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_gemm_group_static(kind, table_host, table_bytes, (uint32_t)count,
                                                          (uint32_t)workgroups, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

int gemm_i8_mfma(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                 int32_t *C, int64_t ldc, void *stream)
{
    const char *name = "gemm_i8_mfma";
    bool empty;
    const int rc = check_gemm_i8(name, M, N, K, A, lda, B, ldb, C, ldc, &empty);
    if (rc != LB_OK || empty)
        return rc;
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_gemm_i8(M, N, K, A, lda, B, ldb, C, ldc, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

size_t gemm_i8_grouped_table_bytes(int64_t count, const lb_i8_problem *problems)
{
    int64_t wg = 0;
    if (i8_group_workgroups("gemm_i8_grouped_table_bytes", count, problems, &wg) != LB_OK)
        return 0;
    return i8_group_table_bytes(count, wg);
}

int gemm_i8_grouped_plan(int64_t count, const lb_i8_problem *problems, void *table, size_t table_bytes,
                         int64_t *workgroups)
{
    const char *name = "gemm_i8_grouped_plan";
    if (!table || !workgroups)
        return fail(LB_EINVAL, "%s: null pointer", name);
    int64_t wg = 0;
    const int rc = i8_group_workgroups(name, count, problems, &wg);
    if (rc != LB_OK)
        return rc;
    const size_t need = i8_group_table_bytes(count, wg);
    if (table_bytes < need)
        return fail(LB_EINVAL, "%s: table_bytes=%zu < %zu", name, table_bytes, need);
    memset(table, 0, need);
    auto *hdr = static_cast<lowbit::I8GroupHeader *>(table);
    auto *recs = reinterpret_cast<lowbit::I8GroupRecord *>(hdr + 1);
    auto *owner = reinterpret_cast<uint32_t *>(recs + count);
    hdr->magic = lowbit::kI8GroupMagic;
    hdr->count = (uint32_t)count;
    hdr->workgroups = (uint32_t)wg;
    uint32_t next = 0;
    constexpr int T = lowbit::kI8GroupTile;
    for (int64_t p = 0; p < count; ++p) {
        const lb_i8_problem &q = problems[p];
        lowbit::I8GroupRecord &r = recs[p];
        r.tile0 = next;
        if (q.M == 0 || q.N == 0)
            continue;  // owns no workgroup; the zeroed record is never read
        r.A = q.A;
        r.B = q.B;
        r.C = q.C;
        r.lda = q.lda;
        r.ldb = q.ldb;
        r.ldc = q.ldc;
        r.M = (int32_t)q.M;
        r.N = (int32_t)q.N;
        r.K = (int32_t)q.K;
        r.nMB = (int32_t)((q.M + T - 1) / T);
        r.mode = lowbit::i8_fetch_mode(q.M, q.N, q.K, q.A, q.lda, q.B, q.ldb, T, T);
        const uint32_t tiles = (uint32_t)r.nMB * (uint32_t)((q.N + T - 1) / T);
        for (uint32_t t = 0; t < tiles; ++t)
            owner[next + t] = (uint32_t)p;
        next += tiles;
    }
    *workgroups = wg;
    return LB_OK;
}

int gemm_i8_grouped(int64_t count, const void *table_dev, int64_t workgroups, void *stream)
{
    const char *name = "gemm_i8_grouped";
    if (count < 0 || workgroups < 0)
        return fail(LB_EINVAL, "%s: count=%lld workgroups=%lld must be >= 0", name, (long long)count,
                    (long long)workgroups);
    if (count > 0x7fffffffLL || workgroups > 0x7fffffffLL)
        return fail(LB_EOVERFLOW, "%s: count=%lld workgroups=%lld exceed 2^31-1", name, (long long)count,
                    (long long)workgroups);
    if (workgroups == 0)
        return LB_OK;
    if (count == 0)
        return fail(LB_EINVAL, "%s: %lld workgroups for no problems", name, (long long)workgroups);
    if (!table_dev || !aligned(table_dev, 16))
        return fail(LB_EINVAL, "%s: table_dev must be a 16-byte aligned device pointer", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_gemm_i8_group(static_cast<const lowbit::I8GroupHeader *>(table_dev),
                                                      (uint32_t)count, (uint32_t)workgroups,
                                                      static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

int gemm_requant(int kind, int out_planes, int64_t M, int64_t N, int64_t K, const uint64_t *Ap, const uint64_t *Bp,
                 const int32_t *lo, const int32_t *hi, uint64_t *Out, void *stream)
{
    const char *name = "gemm_requant";
    if (kind < 0 || kind > 2)
        return fail(LB_EINVAL, "%s: kind=%d must be 0 (BNN), 1 (TNN) or 2 (TBN)", name, kind);
    if (out_planes != 1 && out_planes != 2)
        return fail(LB_EINVAL, "%s: out_planes=%d must be 1 (binary) or 2 (ternary)", name, out_planes);
    if (M < 0 || N < 0)
        return fail(LB_EINVAL, "%s: M=%lld N=%lld must be >= 0", name, (long long)M, (long long)N);
    if (K <= 0)
        return fail(LB_EINVAL, "%s: K=%lld must be >= 1", name, (long long)K);
    if (K > kMaxDepth || M > kMaxExtent || N > kMaxExtent)
        return fail(LB_EOVERFLOW, "%s: M=%lld N=%lld K=%lld exceed 2^31-1", name, (long long)M, (long long)N,
                    (long long)K);
    if (M == 0 || N == 0)
        return LB_OK;
    if (!Ap || !Bp || !Out || !lo || (out_planes == 2 && !hi))
        return fail(LB_EINVAL, "%s: null pointer", name);
    if (!aligned(Ap, 16) || !aligned(Bp, 16) || !aligned(Out, 16) || !aligned(lo, 4) || !aligned(hi, 4))
        return fail(LB_EINVAL, "%s: packed operands must be 16-byte aligned, thresholds 4-byte aligned", name);
    if (packed_bytes(N, M, out_planes == 2 ? 16 : 8) == 0)
        return fail(LB_EOVERFLOW, "%s: output size overflows", name);
    const int64_t KW = (K + 63) / 64;
    int count = 0;
    const lowbit::GemmVariant *tab = lowbit::gemm_variants(kind, &count);
    // lanes own rows of C (output channels): a wave-wide vote then yields one packed depth word of the output
    lowbit::GemmArgs a;
    a.Sp = reinterpret_cast<const uint32_t *>(Bp);
    a.rowsS = (int)N;
    a.Vp = reinterpret_cast<const uint32_t *>(Ap);
    a.rowsV = (int)M;
    a.KW = (int)KW;
    a.K = (int)K;
    a.C = nullptr;
    a.ldc = 0;
    a.stream = static_cast<hipStream_t>(stream);
    a.q_lo = lo;
    a.q_hi = hi;
    a.q_out = Out;
    a.q_planes = out_planes;
    const int fv = forced_variant(kind);
    const int v = (fv >= 0 && fv < count) ? fv : choose_variant(tab, count, a.rowsS, a.rowsV, a.KW, true);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = tab[v].launch_transposed(a);
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

int gemm_u8_mfma(int64_t M, int64_t N, int64_t K, const uint8_t *A, int64_t lda, const uint8_t *B, int64_t ldb,
                 int32_t zA, int32_t zB, int32_t *C, int64_t ldc, void *stream)
{
    const char *name = "gemm_u8_mfma";
    if (M < 0 || N < 0)
        return fail(LB_EINVAL, "%s: M=%lld N=%lld must be >= 0", name, (long long)M, (long long)N);
    if (K <= 0)
        return fail(LB_EINVAL, "%s: K=%lld must be >= 1", name, (long long)K);
    if (zA < 0 || zA > 255 || zB < 0 || zB > 255)
        return fail(LB_EINVAL, "%s: zero points zA=%d zB=%d must lie in [0, 255]", name, zA, zB);
    // |(a - zA)(b - zB)| <= 255^2, so the int32 sum is safe up to K = floor((2^31 - 1) / 255^2)
    if (K > 33025)
        return fail(LB_EOVERFLOW, "%s: K=%lld exceeds 33025 (int32 accumulation of 8-bit products)", name,
                    (long long)K);
    if (M > kMaxExtent || N > kMaxExtent)
        return fail(LB_EOVERFLOW, "%s: M=%lld N=%lld exceed 2^31-1", name, (long long)M, (long long)N);
    if (M == 0 || N == 0)
        return LB_OK;
    if (!A || !B || !C)
        return fail(LB_EINVAL, "%s: null pointer", name);
    if (lda < K || ldb < N || ldc < N)
        return fail(LB_EINVAL, "%s: lda=%lld ldb=%lld ldc=%lld too small", name, (long long)lda, (long long)ldb,
                    (long long)ldc);
    if (lda > INT64_MAX / M || ldb > INT64_MAX / K || ldc > INT64_MAX / M / 4)
        return fail(LB_EOVERFLOW, "%s: matrix extent overflows", name);
    if (!aligned(C, 4))
        return fail(LB_EINVAL, "%s: C must be 4-byte aligned", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e =
        lowbit::launch_gemm_u8(M, N, K, A, lda, B, ldb, zA, zB, C, ldc, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

int im2col_packed(const uint64_t *Fp, int planes, int64_t batch, int64_t H, int64_t W, int64_t C, int kh, int kw,
                  int stride_h, int stride_w, int pad_h, int pad_w, uint64_t *Bp, void *stream)
{
    const char *name = "im2col_packed";
    if (planes != 1 && planes != 2)
        return fail(LB_EINVAL, "%s: planes=%d must be 1 (binary) or 2 (ternary)", name, planes);
    lowbit::Im2colGeom g;
    bool empty;
    const int rc = check_conv_geom(name, batch, H, W, C, kh, kw, stride_h, stride_w, pad_h, pad_w, &g, &empty);
    if (rc != LB_OK || empty)
        return rc;
    if (!Fp || !Bp)
        return fail(LB_EINVAL, "%s: null pointer", name);
    if (!aligned(Fp, 16) || !aligned(Bp, 16))
        return fail(LB_EINVAL, "%s: operands must be 16-byte aligned", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_im2col_packed(planes, Fp, Bp, g, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

int conv_gemm(int kind, int64_t M, const uint64_t *Ap, const uint64_t *Fp, int64_t batch, int64_t H, int64_t W,
              int64_t C, int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w, int32_t *Cout, int64_t ldc,
              void *stream)
{
    const char *name = "conv_gemm";
    if (kind < 0 || kind > 2)
        return fail(LB_EINVAL, "%s: kind=%d must be 0 (BNN), 1 (TNN) or 2 (TBN)", name, kind);
    lowbit::Im2colGeom g;
    bool empty;
    int rc = check_conv_geom(name, batch, H, W, C, kh, kw, stride_h, stride_w, pad_h, pad_w, &g, &empty);
    if (rc != LB_OK)
        return rc;
    if (M < 0)
        return fail(LB_EINVAL, "%s: M=%lld must be >= 0", name, (long long)M);
    if (kind == lowbit::KIND_TBN)
        return fail(LB_EUNSUPPORTED,
                    "%s: the ternary-binary kernel keeps the binary operand (here the feature map) in scalar registers, "
                    "where it cannot be gathered; use im2col_packed + gemm_tbn",
                    name);
    if (empty || M == 0)
        return LB_OK;
    const int64_t N = batch * g.OH * g.OW, K = (int64_t)kh * kw * C;  // both bounded by check_conv_geom
    if (N > kMaxExtent)
        return fail(LB_EOVERFLOW, "%s: %lld output pixels exceed 2^31-1", name, (long long)N);
    rc = check_gemm(name, M, N, K, Ap, Fp, Cout, ldc, &empty);
    if (rc != LB_OK)
        return rc;
    if (const int rc_dev = check_device(name))
        return rc_dev;
    int count = 0;
    const lowbit::GemmVariant *tab = lowbit::gemm_variants(kind, &count);
    lowbit::GemmArgs a;
    a.Sp = reinterpret_cast<const uint32_t *>(Ap);
    a.rowsS = (int)M;
    a.Vp = reinterpret_cast<const uint32_t *>(Fp);
    a.rowsV = (int)N;
    a.KW = (int)(K / 64);
    a.K = (int)K;
    a.C = Cout;
    a.ldc = ldc;
    a.stream = static_cast<hipStream_t>(stream);
    const int fv = forced_variant(kind);
    const int v = (fv >= 0 && fv < count) ? fv : choose_variant(tab, count, a.rowsS, a.rowsV, a.KW, true);
    const hipError_t e = tab[v].launch_conv(a, g);
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

size_t packed_u4_bytes(int64_t rows, int64_t K)
{
    if (rows <= 0 || K <= 0 || rows > kMaxExtent || K > kMaxDepth)
        return 0;
    const int64_t RB = (rows + 31) / 32, KB = 2 * ((K + 127) / 128);
    return (size_t)(RB * KB * 1536);  // < 2^26 * 2^25 * 2^11
}

int pack_u4(const uint8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, void *dst, int32_t *sums,
            void *stream)
{
    const char *name = "pack_u4";
    bool nothing, k_contig;
    const int rc = check_pack(name, src, rows, K, stride_r, stride_k, dst, kU4MaxDepth, &nothing, &k_contig);
    if (rc != LB_OK || nothing)
        return rc;
    if (!sums || !aligned(sums, 4))
        return fail(LB_EINVAL, "%s: sums must be a 4-byte aligned device pointer", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_pack_u4(src, rows, K, k_contig ? stride_r : 1, k_contig ? 1 : stride_k,
                                                static_cast<uint8_t *>(dst), sums, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

int gemm_u4_mfma(int64_t M, int64_t N, int64_t K, const void *Ap, const int32_t *sumA, const void *Bp,
                 const int32_t *sumB, int32_t zA, int32_t zB, int32_t *C, int64_t ldc, void *stream)
{
    const char *name = "gemm_u4_mfma";
    if (M < 0 || N < 0)
        return fail(LB_EINVAL, "%s: M=%lld N=%lld must be >= 0", name, (long long)M, (long long)N);
    if (K <= 0)
        return fail(LB_EINVAL, "%s: K=%lld must be >= 1", name, (long long)K);
    if (zA < 0 || zA > 15 || zB < 0 || zB > 15)
        return fail(LB_EINVAL, "%s: zero points zA=%d zB=%d must lie in [0, 15]", name, zA, zB);
    // 15 * 15 * K < 2^24 keeps every fp32 partial sum of the integer products exact
    if (K > kU4MaxDepth)
        return fail(LB_EOVERFLOW, "%s: K=%lld exceeds %lld (exact fp32 accumulation of 4-bit products)", name,
                    (long long)K, (long long)kU4MaxDepth);
    if (M > kMxMaxExtent || N > kMxMaxExtent)
        return fail(LB_EOVERFLOW, "%s: M=%lld N=%lld exceed 2^31-256", name, (long long)M, (long long)N);
    if (M == 0 || N == 0)
        return LB_OK;
    if (!Ap || !Bp || !sumA || !sumB || !C)
        return fail(LB_EINVAL, "%s: null pointer", name);
    if (ldc < N)
        return fail(LB_EINVAL, "%s: ldc=%lld < N=%lld", name, (long long)ldc, (long long)N);
    if (ldc > INT64_MAX / M / 4)
        return fail(LB_EOVERFLOW, "%s: M*ldc overflows", name);
    if (!aligned(Ap, 16) || !aligned(Bp, 16) || !aligned(sumA, 4) || !aligned(sumB, 4) || !aligned(C, 4))
        return fail(LB_EINVAL, "%s: packed operands must be 16-byte aligned, sums and C 4-byte aligned", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e =
        lowbit::launch_gemm_u4(M, N, K, static_cast<const uint8_t *>(Ap), sumA, static_cast<const uint8_t *>(Bp), sumB,
                               zA, zB, C, ldc, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

size_t packed_t4_bytes(int64_t rows, int64_t K)
{
    if (rows <= 0 || K <= 0 || rows > kMaxExtent || K > kT4MaxDepth)
        return 0;
    const int64_t RB = (rows + 31) / 32, KB = 2 * ((K + 127) / 128);
    return (size_t)(RB * KB * 1024);
}

int pack_t4(const int8_t *src, int64_t rows, int64_t K, int64_t stride_r, int64_t stride_k, void *dst, void *stream)
{
    const char *name = "pack_t4";
    bool nothing, k_contig;
    const int rc = check_pack(name, src, rows, K, stride_r, stride_k, dst, kT4MaxDepth, &nothing, &k_contig);
    if (rc != LB_OK || nothing)
        return rc;
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_pack_t4(src, rows, K, k_contig ? stride_r : 1, k_contig ? 1 : stride_k,
                                                static_cast<uint8_t *>(dst), static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

int gemm_t4_mfma(int64_t M, int64_t N, int64_t K, const void *Ap, const void *Bp, int32_t *C, int64_t ldc, void *stream)
{
    const char *name = "gemm_t4_mfma";
    if (M < 0 || N < 0)
        return fail(LB_EINVAL, "%s: M=%lld N=%lld must be >= 0", name, (long long)M, (long long)N);
    if (K <= 0)
        return fail(LB_EINVAL, "%s: K=%lld must be >= 1", name, (long long)K);
    // |sum| <= K < 2^24 keeps every fp32 partial sum exact
    if (K > kT4MaxDepth)
        return fail(LB_EOVERFLOW, "%s: K=%lld exceeds %lld (exact fp32 accumulation)", name, (long long)K,
                    (long long)kT4MaxDepth);
    if (M > kMxMaxExtent || N > kMxMaxExtent)
        return fail(LB_EOVERFLOW, "%s: M=%lld N=%lld exceed 2^31-256", name, (long long)M, (long long)N);
    if (M == 0 || N == 0)
        return LB_OK;
    if (!Ap || !Bp || !C)
        return fail(LB_EINVAL, "%s: null pointer", name);
    if (ldc < N)
        return fail(LB_EINVAL, "%s: ldc=%lld < N=%lld", name, (long long)ldc, (long long)N);
    if (ldc > INT64_MAX / M / 4)
        return fail(LB_EOVERFLOW, "%s: M*ldc overflows", name);
    if (!aligned(Ap, 16) || !aligned(Bp, 16) || !aligned(C, 4))
        return fail(LB_EINVAL, "%s: packed operands must be 16-byte aligned, C 4-byte aligned", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_gemm_t4(M, N, K, static_cast<const uint8_t *>(Ap), static_cast<const uint8_t *>(Bp),
                                                C, ldc, static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

size_t lb_calib_sink_bytes(void) { return (size_t)lowbit::calib_grid_blocks() * 2 * 256 * 4; }

int64_t lb_calib_valu_lane_instr(int mix, int64_t iters, int waves_per_simd)
{
    if (mix < 0 || mix >= lowbit::CALIB_NUM_MIXES || iters <= 0 || iters > (1 << 24) || waves_per_simd < 1 ||
        waves_per_simd > 8)
        return 0;
    return lowbit::calib_valu_lane_instr(mix, iters, waves_per_simd);
}

size_t lb_calib_clocks_bytes(void) { return (size_t)lowbit::calib_grid_blocks() * 2 * 8; }

int lb_calib_wall_clock_khz(void) { return lowbit::calib_wall_clock_khz(); }

int lb_calib_valu(int mix, int64_t iters, int waves_per_simd, void *sink, void *clocks, void *stream)
{
    const char *name = "lb_calib_valu";
    if (mix < 0 || mix >= lowbit::CALIB_NUM_MIXES)
        return fail(LB_EINVAL, "%s: mix=%d must lie in [0, %d)", name, mix, (int)lowbit::CALIB_NUM_MIXES);
    if (iters <= 0 || iters > (1 << 24))
        return fail(LB_EINVAL, "%s: iters=%lld must lie in [1, 2^24]", name, (long long)iters);
    if (waves_per_simd < 1 || waves_per_simd > 8)
        return fail(LB_EINVAL, "%s: waves_per_simd=%d must lie in [1, 8]", name, waves_per_simd);
    if (!sink || !aligned(sink, 4))
        return fail(LB_EINVAL, "%s: sink must be a 4-byte aligned device buffer", name);
    if (!aligned(clocks, 8))
        return fail(LB_EINVAL, "%s: clocks must be NULL or an 8-byte aligned device buffer", name);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_calib_valu(mix, (int)iters, waves_per_simd, static_cast<uint32_t *>(sink),
                                                   static_cast<unsigned long long *>(clocks),
                                                   static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

int lb_calib_stream(int mode, const void *src, void *dst, int64_t bytes, int blocks, void *sink, void *stream)
{
    const char *name = "lb_calib_stream";
    if (mode < 0 || mode > 2)
        return fail(LB_EINVAL, "%s: mode=%d must be 0 (read), 1 (write) or 2 (copy)", name, mode);
    if (bytes <= 0 || bytes % 16 != 0)
        return fail(LB_EINVAL, "%s: bytes=%lld must be a positive multiple of 16", name, (long long)bytes);
    if (blocks < 0 || blocks > 2 * lowbit::calib_grid_blocks())
        return fail(LB_EINVAL, "%s: blocks=%d must lie in [0, %d]", name, blocks, 2 * lowbit::calib_grid_blocks());
    if ((mode != 1 && (!src || !aligned(src, 16))) || (mode != 0 && (!dst || !aligned(dst, 16))) ||
        (mode == 0 && (!sink || !aligned(sink, 4))))
        return fail(LB_EINVAL, "%s: missing or misaligned buffer for mode %d", name, mode);
    if (const int rc_dev = check_device(name))
        return rc_dev;
    const hipError_t e = lowbit::launch_calib_stream(mode, src, dst, bytes, blocks, static_cast<uint32_t *>(sink),
                                                     static_cast<hipStream_t>(stream));
    if (e != hipSuccess)
        return fail(LB_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LB_OK;
}

const char *lb_describe_plan(int kind, int64_t M, int64_t N, int64_t K, int c16)
{
    thread_local char text[160];
    if (kind < 0 || kind > 2 || M <= 0 || N <= 0 || K <= 0 || K > kMaxDepth || M > kMaxExtent || N > kMaxExtent)
        return nullptr;
    const GemmPlan p = plan_gemm(kind, M, N, K, c16 != 0);
    static const char *const kinds[] = {"bnn", "tnn", "tbn", "tbn (ternary operand on the scalar side / in LDS)"};
    if (p.path == GemmPlan::SKINNY) {
        snprintf(text, sizeof(text), "%s depth-split-across-lanes kernel, %s streamed", kinds[p.kind],
                 p.transposed ? "B" : "A");
    } else if (p.path == GemmPlan::SPLIT) {
        snprintf(text, sizeof(text), "%s tiled kernel, %d depth ranges added into a cleared C", kinds[p.kind], p.nsplit);
    } else {
        int count = 0;
        const lowbit::GemmVariant *tab = lowbit::gemm_variants(p.kind, &count);
        snprintf(text, sizeof(text), "%s tiled kernel [%s], %s on the scalar side", kinds[p.kind], tab[p.variant].name,
                 p.transposed ? "B" : "A");
    }
    return text;
}

int lb_set_variant(int op, int variant)
{
    int count = 0;
    if (op == 4) {
        if (variant < -1 || variant >= kI8Instances)
            return fail(LB_EINVAL, "lb_set_variant: int8 tile %d out of range", variant);
        lowbit::i8_force_tile(variant);
        return LB_OK;
    }
    if (op == 5) {
        if (variant < -1 || variant >= lowbit::u4_num_instances())
            return fail(LB_EINVAL, "lb_set_variant: 4-bit instance %d out of range", variant);
        lowbit::u4_force_instance(variant);
        return LB_OK;
    }
    if (op == 3) {
        if (variant < -1 || variant >= lowbit::skinny_num_configs())
            return fail(LB_EINVAL, "lb_set_variant: skinny config %d out of range", variant);
        lowbit::skinny_force_config(variant);
        return LB_OK;
    }
    if (op < 0 || op > 2 || !lowbit::gemm_variants(op, &count))
        return fail(LB_EINVAL, "lb_set_variant: op=%d out of range", op);
    if (variant < -1 || variant >= count)
        return fail(LB_EINVAL, "lb_set_variant: variant=%d out of range [-1,%d)", variant, count);
    g_forced[op].store(variant, std::memory_order_relaxed);
    return LB_OK;
}

int lb_num_variants(int op)
{
    int count = 0;
    if (op == 3)
        return lowbit::skinny_num_configs();
    if (op == 4)
        return kI8Instances;
    if (op == 5)
        return lowbit::u4_num_instances();
    if (op < 0 || op > 2)
        return 0;
    lowbit::gemm_variants(op, &count);
    return count;
}

const char *lb_variant_name(int op, int variant)
{
    int count = 0;
    if (op < 0 || op > 2)
        return nullptr;
    const lowbit::GemmVariant *tab = lowbit::gemm_variants(op, &count);
    if (variant < 0 || variant >= count)
        return nullptr;
    return tab[variant].name;
}

}  // extern "C"
