// Host-only exerciser of the C ABI's validation, planning and dispatch logic, meant to be built with
// AddressSanitizer and UndefinedBehaviorSanitizer on the HOST side and run without a GPU (tests/test_sanitizers.py).
// Every table the library writes goes into a heap block of exactly the advertised size, so a write past it, a read of
// a too-short problem array or an overflow in the index arithmetic ends the program with a sanitizer report.
// No kernel is launched: calls with valid arguments stop at the device check (no device here) and return an error.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "lowbit_gemm.h"
#include "lowbit_gemm_bench.h"

static int g_failures = 0;

#define EXPECT(cond)                                                                     \
    do {                                                                                 \
        if (!(cond)) {                                                                   \
            std::printf("FAILED %s:%d: %s   [last error: %s]\n", __FILE__, __LINE__, #cond, lb_last_error()); \
            ++g_failures;                                                                \
        }                                                                                \
    } while (0)

// Addresses that are never dereferenced on the host: the planning calls only store them.
static uint64_t *fake_u64(uintptr_t n) { return reinterpret_cast<uint64_t *>(uintptr_t(0x100000000ULL) + n * 0x1000000ULL); }
static int8_t *fake_i8(uintptr_t n, uintptr_t odd = 0) { return reinterpret_cast<int8_t *>(uintptr_t(0x200000000ULL) + n * 0x1000000ULL + odd); }
static int32_t *fake_i32(uintptr_t n) { return reinterpret_cast<int32_t *>(uintptr_t(0x300000000ULL) + n * 0x1000000ULL); }

static const int64_t kBig = INT64_MAX;

static void size_helpers()
{
    EXPECT(packed_binary_bytes(3, 65) == 3 * 2 * 8);
    EXPECT(packed_ternary_bytes(3, 65) == 3 * 2 * 16);
    EXPECT(packed_binary_bytes(0, 64) == 0);
    EXPECT(packed_binary_bytes(-1, 64) == 0 && packed_ternary_bytes(5, -3) == 0);
    EXPECT(packed_binary_bytes(kBig, kBig) == 0 && packed_ternary_bytes(kBig, 64) == 0);
    EXPECT(packed_ternary_bytes(kBig / 16, 64) == 0 || packed_ternary_bytes(kBig / 16, 64) % 16 == 0);
    EXPECT(packed_u4_bytes(-1, 5) == 0 && packed_u4_bytes(kBig, kBig) == 0 && packed_u4_bytes(33, 129) > 0);
    EXPECT(packed_t4_bytes(-1, 5) == 0 && packed_t4_bytes(kBig, kBig) == 0 && packed_t4_bytes(33, 129) > 0);
    EXPECT(lb_format_version() == LB_FORMAT_VERSION);
}

static void arch_names()
{
    EXPECT(lb_arch_supported("gfx950") == 1);
    EXPECT(lb_arch_supported("gfx950:sramecc+:xnack-") == 1);
    EXPECT(lb_arch_supported("gfx9500") == 0);
    EXPECT(lb_arch_supported("gfx942") == 0);
    EXPECT(lb_arch_supported("gfx95") == 0);
    EXPECT(lb_arch_supported("") == 0);
    EXPECT(lb_arch_supported(nullptr) == 0);
    char *exact = static_cast<char *>(std::malloc(7));  // "gfx950" + NUL in a block of exactly that size
    std::memcpy(exact, "gfx950", 7);
    EXPECT(lb_arch_supported(exact) == 1);
    std::free(exact);
    char *unterminated_prefix = static_cast<char *>(std::malloc(4));
    std::memcpy(unterminated_prefix, "gfx", 4);
    EXPECT(lb_arch_supported(unterminated_prefix) == 0);
    std::free(unterminated_prefix);
}

static void single_call_validation()
{
    uint64_t *A = fake_u64(1), *B = fake_u64(2);
    int32_t *C = fake_i32(1);
    EXPECT(gemm_tnn(-1, 4, 64, A, B, C, 4, nullptr) == LB_EINVAL);
    EXPECT(gemm_tnn(4, 4, 0, A, B, C, 4, nullptr) == LB_EINVAL);
    EXPECT(gemm_bnn(4, 4, 64, nullptr, B, C, 4, nullptr) == LB_EINVAL);
    EXPECT(gemm_tbn(4, 4, 64, A, B, C, 3, nullptr) == LB_EINVAL);
    EXPECT(gemm_tnn(4, 4, (int64_t(1) << 31), A, B, C, 4, nullptr) == LB_EOVERFLOW);
    EXPECT(gemm_tnn(kBig, kBig, 64, A, B, C, kBig, nullptr) == LB_EOVERFLOW);
    EXPECT(gemm_tnn(4, 4, 64, A, B, C, kBig, nullptr) == LB_EOVERFLOW);
    EXPECT(gemm_tnn(4, 4, 64, reinterpret_cast<uint64_t *>(uintptr_t(A) + 8), B, C, 4, nullptr) == LB_EINVAL);
    EXPECT(std::strlen(lb_last_error()) > 0);
    EXPECT(gemm_tnn(0, 4, 64, nullptr, nullptr, nullptr, 0, nullptr) == LB_OK);  // empty product: nothing to do
    EXPECT(gemm_c16(1, 4, 4, 32768, A, B, reinterpret_cast<int16_t *>(C), 4, nullptr) < 0);
    EXPECT(gemm_c16(7, 4, 4, 64, A, B, reinterpret_cast<int16_t *>(C), 4, nullptr) == LB_EINVAL);
    // valid arguments: stops at the device check on a machine without a gfx950 (any error code), never crashes
    const int rc = gemm_tnn(4, 4, 64, A, B, C, 4, nullptr);
    EXPECT(rc == LB_EHIP || rc == LB_EUNSUPPORTED);

    int8_t *src = fake_i8(1);
    EXPECT(pack_ternary(nullptr, 4, 64, 64, 1, A, nullptr) == LB_EINVAL);
    EXPECT(pack_ternary(src, -4, 64, 64, 1, A, nullptr) == LB_EINVAL);
    EXPECT(pack_binary(src, 4, 64, 64, 2, A, nullptr) < 0);
    EXPECT(pack_binary(src, kBig, kBig, kBig, 1, A, nullptr) < 0);
    EXPECT(pack_ternary(src, kBig / 2, 64, 64, 1, A, nullptr) < 0);

    EXPECT(gemm_i8_mfma(4, 4, 64, nullptr, 64, src, 4, C, 4, nullptr) == LB_EINVAL);
    EXPECT(gemm_i8_mfma(4, 4, 64, src, 63, src, 4, C, 4, nullptr) == LB_EINVAL);
    EXPECT(gemm_i8_mfma(kBig, kBig, kBig, src, kBig, src, kBig, C, kBig, nullptr) < 0);
    EXPECT(gemm_u8_mfma(4, 4, 64, reinterpret_cast<uint8_t *>(src), 64, reinterpret_cast<uint8_t *>(src), 4, 300, 0, C, 4,
                        nullptr) < 0);

    // convolution geometry
    EXPECT(conv_gemm(1, 8, A, B, 1, 8, 8, 64, 3, 3, 1, 1, 1, 1, C, 63, nullptr) == LB_EINVAL);   // ldc < pixels
    EXPECT(conv_gemm(1, 8, A, B, 1, 8, 8, 65, 3, 3, 1, 1, 1, 1, C, 64, nullptr) < 0);            // channels % 64
    EXPECT(conv_gemm(1, 8, A, B, 1, 8, 8, 64, 0, 3, 1, 1, 1, 1, C, 64, nullptr) == LB_EINVAL);
    EXPECT(conv_gemm(1, 8, A, B, 1, 8, 8, 64, 3, 3, 0, 1, 1, 1, C, 64, nullptr) == LB_EINVAL);
    EXPECT(conv_gemm(1, 8, A, B, 1, 2, 2, 64, 5, 5, 1, 1, 0, 0, C, 64, nullptr) == LB_OK);       // no output pixel: no-op
    EXPECT(conv_gemm(2, 8, A, B, 1, 8, 8, 64, 3, 3, 1, 1, 1, 1, C, 64, nullptr) == LB_EUNSUPPORTED);
    EXPECT(conv_gemm(1, 8, A, B, kBig, kBig, kBig, 64, 3, 3, 1, 1, 1, 1, C, kBig, nullptr) < 0);
    EXPECT(conv_gemm(1, 8, A, B, 1 << 20, 1 << 20, 1 << 20, 1 << 20, 3, 3, 1, 1, 1, 1, C, kBig, nullptr) < 0);
    EXPECT(im2col_packed(A, 2, kBig, kBig, kBig, 64, 3, 3, 1, 1, 1, 1, B, nullptr) < 0);
    EXPECT(im2col_packed(A, 3, 1, 8, 8, 64, 3, 3, 1, 1, 1, 1, B, nullptr) == LB_EINVAL);
}

static void describe_plans()
{
    static const int64_t dims[] = {0, 1, 7, 8, 9, 31, 32, 33, 63, 64, 65, 72, 360, 1024, 4096, 50176, 131072, 1 << 20,
                                   (int64_t(1) << 31) - 1, int64_t(1) << 31, kBig};
    static const int64_t depths[] = {0, 1, 63, 64, 65, 576, 2048, 4608, 16384, 65536, 32767, 32768, (int64_t(1) << 31) - 1,
                                     int64_t(1) << 31, kBig};
    size_t described = 0;
    for (int kind = -1; kind <= 3; ++kind)
        for (int64_t M : dims)
            for (int64_t N : dims)
                for (int64_t K : depths)
                    for (int c16 = 0; c16 <= 1; ++c16) {
                        const char *s = lb_describe_plan(kind, M, N, K, c16);
                        const bool valid = kind >= 0 && kind <= 2 && M >= 1 && N >= 1 && K >= 1 && M < (int64_t(1) << 31) &&
                                           N < (int64_t(1) << 31) && K < (int64_t(1) << 31);
                        EXPECT((s != nullptr) == valid);  // NULL is the documented answer for an invalid request
                        if (s)
                            described += std::strlen(s) > 0;
                    }
    EXPECT(described > 1000);
    for (int op = -1; op <= 6; ++op) {
        const int n = lb_num_variants(op);
        for (int v = -2; v <= n + 1; ++v) {
            const char *name = lb_variant_name(op, v);  // NULL outside the tile tables
            EXPECT(name == nullptr || std::strlen(name) > 0);
            EXPECT((name != nullptr) == (op >= 0 && op <= 2 && v >= 0 && v < n));
            const int rc = lb_set_variant(op, v);
            EXPECT(rc == LB_OK || rc == LB_EINVAL);
        }
        lb_set_variant(op, -1);
    }
}

template <class Problem, class Bytes, class Plan>
static void plan_exact(const char *what, std::vector<Problem> &ps, Bytes bytes_fn, Plan plan_fn, bool expect_ok)
{
    // the problem array itself in a block of exactly count entries
    Problem *arr = static_cast<Problem *>(std::malloc(ps.size() * sizeof(Problem) + 1));
    std::memcpy(arr, ps.data(), ps.size() * sizeof(Problem));
    const size_t bytes = bytes_fn((int64_t)ps.size(), arr);
    if (!expect_ok) {
        EXPECT(bytes == 0);
        int64_t wg = -7;
        unsigned char dummy[16];
        EXPECT(plan_fn((int64_t)ps.size(), arr, dummy, sizeof(dummy), &wg) < 0);
        std::free(arr);
        return;
    }
    EXPECT(bytes > 0 && bytes % 16 == 0);
    unsigned char *table = static_cast<unsigned char *>(std::malloc(bytes));
    int64_t wg = -1;
    const int rc = plan_fn((int64_t)ps.size(), arr, table, bytes, &wg);
    EXPECT(rc == LB_OK);
    EXPECT(wg >= 0);
    // one byte short: refused, nothing written beyond the block
    unsigned char *small = static_cast<unsigned char *>(std::malloc(bytes - 1));
    int64_t wg2 = -1;
    EXPECT(plan_fn((int64_t)ps.size(), arr, small, bytes - 1, &wg2) == LB_EINVAL);
    EXPECT(plan_fn((int64_t)ps.size(), arr, nullptr, bytes, &wg2) == LB_EINVAL);
    EXPECT(plan_fn((int64_t)ps.size(), arr, table, bytes, nullptr) == LB_EINVAL);
    // planning is deterministic: same bytes again
    unsigned char *again = static_cast<unsigned char *>(std::malloc(bytes));
    EXPECT(plan_fn((int64_t)ps.size(), arr, again, bytes, &wg2) == LB_OK && wg2 == wg);
    EXPECT(std::memcmp(table, again, bytes) == 0);
    std::printf("  %-34s %4zu problems  %7zu table bytes  %6lld workgroups\n", what, ps.size(), bytes, (long long)wg);
    std::free(again);
    std::free(small);
    std::free(table);
    std::free(arr);
}

static void grouped_popcount()
{
    for (int kind = 0; kind <= 2; ++kind) {
        auto bytes_fn = [kind](int64_t n, const lb_gemm_problem *p) { return gemm_grouped_table_bytes(kind, n, p); };
        auto plan_fn = [kind](int64_t n, const lb_gemm_problem *p, void *t, size_t b, int64_t *wg) {
            return gemm_grouped_plan(kind, n, p, t, b, wg);
        };
        std::vector<lb_gemm_problem> grid;  // the 4 x 4 x 4 shape grid of Section IV-B
        uintptr_t id = 0;
        for (int64_t H : {72, 120, 240, 360})
            for (int64_t W : {24, 48, 72, 96})
                for (int64_t D : {128, 256, 384, 512})
                    grid.push_back({H, W, D, fake_u64(++id), fake_u64(++id), fake_i32(id), W});
        plan_exact("shape grid of Section IV-B", grid, bytes_fn, plan_fn, true);

        std::vector<lb_gemm_problem> ragged = {
            {1, 1, 1, fake_u64(1), fake_u64(2), fake_i32(3), 1},        {17, 65, 65, fake_u64(4), fake_u64(5), fake_i32(6), 70},
            {0, 9, 64, nullptr, nullptr, nullptr, 0},                   {9, 0, 64, nullptr, nullptr, nullptr, 0},
            {257, 2, 64, fake_u64(7), fake_u64(8), fake_i32(9), 2},     {2, 257, 640, fake_u64(10), fake_u64(11), fake_i32(12), 300},
            {3000, 5000, 100000, fake_u64(13), fake_u64(14), fake_i32(15), 5000}};
        plan_exact("ragged, empty and large problems", ragged, bytes_fn, plan_fn, true);

        std::vector<lb_gemm_problem> none;
        {
            const size_t b = gemm_grouped_table_bytes(kind, 0, nullptr);
            int64_t wg = -1;
            unsigned char *t = static_cast<unsigned char *>(std::malloc(b ? b : 1));
            EXPECT(gemm_grouped_plan(kind, 0, nullptr, t, b, &wg) == LB_OK && wg == 0);
            EXPECT(gemm_grouped(kind, 0, t, 0, nullptr) == LB_OK);
            std::free(t);
        }

        std::vector<lb_gemm_problem> bad = grid;
        bad[40].ldc = bad[40].N - 1;
        plan_exact("bad ldc", bad, bytes_fn, plan_fn, false);
        bad = grid;
        bad[63].K = int64_t(1) << 31;
        plan_exact("depth overflow", bad, bytes_fn, plan_fn, false);
        bad = grid;
        bad[0].Ap = nullptr;
        plan_exact("null operand", bad, bytes_fn, plan_fn, false);
        bad = grid;
        bad[5].Bp = reinterpret_cast<const uint64_t *>(uintptr_t(bad[5].Bp) + 4);
        plan_exact("misaligned operand", bad, bytes_fn, plan_fn, false);
        bad = grid;
        for (auto &q : bad) {
            q.M = (int64_t(1) << 31) - 1;
            q.N = (int64_t(1) << 31) - 1;
            q.ldc = q.N;
        }
        plan_exact("too many workgroups", bad, bytes_fn, plan_fn, false);

        // the allocation-free variant: host-side checks come before any device work
        const size_t gb = bytes_fn((int64_t)grid.size(), grid.data());
        unsigned char *t = static_cast<unsigned char *>(std::malloc(gb));
        int64_t wg = 0;
        EXPECT(plan_fn((int64_t)grid.size(), grid.data(), t, gb, &wg) == LB_OK);
        EXPECT(gemm_grouped_static(kind, (int64_t)grid.size(), nullptr, gb, wg, nullptr) == LB_EINVAL);
        EXPECT(gemm_grouped_static(kind, (int64_t)grid.size(), t, gb - 16, wg, nullptr) == LB_EINVAL);
        EXPECT(gemm_grouped_static(kind, (int64_t)grid.size() + 1, t, gb, wg, nullptr) == LB_EINVAL);
        EXPECT(gemm_grouped_static((kind + 1) % 3, (int64_t)grid.size(), t, gb, wg, nullptr) == LB_EINVAL);
        EXPECT(gemm_grouped_static(kind, (int64_t)grid.size(), t, gb, wg + 1, nullptr) == LB_EINVAL);
        const int rc = gemm_grouped_static(kind, (int64_t)grid.size(), t, gb, wg, nullptr);
        EXPECT(rc == LB_EHIP || rc == LB_EUNSUPPORTED);  // valid: stops at the device check here
        std::free(t);
        // a table beyond the array inside the library
        std::vector<lb_gemm_problem> many(2000, grid[63]);
        const size_t mb = bytes_fn((int64_t)many.size(), many.data());
        EXPECT(mb > gemm_grouped_static_max_bytes());
        unsigned char *mt = static_cast<unsigned char *>(std::malloc(mb));
        EXPECT(plan_fn((int64_t)many.size(), many.data(), mt, mb, &wg) == LB_OK);
        EXPECT(gemm_grouped_static(kind, (int64_t)many.size(), mt, mb, wg, nullptr) == LB_EUNSUPPORTED);
        std::free(mt);
    }
    EXPECT(gemm_grouped_table_bytes(3, 0, nullptr) == 0);
    EXPECT(gemm_grouped_table_bytes(1, -1, nullptr) == 0);
    EXPECT(gemm_grouped_table_bytes(1, 5, nullptr) == 0);
    EXPECT(gemm_grouped_table_bytes(1, int64_t(1) << 40, reinterpret_cast<lb_gemm_problem *>(fake_u64(1))) == 0);
}

static void grouped_i8()
{
    auto bytes_fn = [](int64_t n, const lb_i8_problem *p) { return gemm_i8_grouped_table_bytes(n, p); };
    auto plan_fn = [](int64_t n, const lb_i8_problem *p, void *t, size_t b, int64_t *wg) {
        return gemm_i8_grouped_plan(n, p, t, b, wg);
    };
    std::vector<lb_i8_problem> grid;
    uintptr_t id = 0;
    for (int64_t H : {72, 120, 240, 360})
        for (int64_t W : {24, 48, 72, 96})
            for (int64_t D : {128, 256, 384, 512}) {
                ++id;
                grid.push_back({H, W, D, fake_i8(id), D, fake_i8(id + 100), W, fake_i32(id), W});
            }
    plan_exact("8-bit: shape grid of Section IV-B", grid, bytes_fn, plan_fn, true);
    std::vector<lb_i8_problem> ragged = {
        {1, 1, 1, fake_i8(1, 1), 1, fake_i8(2, 3), 1, fake_i32(3), 1},
        {65, 67, 66, fake_i8(4, 1), 69, fake_i8(5, 3), 68, fake_i32(6), 70},
        {0, 9, 64, nullptr, 0, nullptr, 0, nullptr, 0},
        {128, 128, 131071, fake_i8(7), 131071, fake_i8(8), 128, fake_i32(9), 128},
        {100, 16, 48, fake_i8(10), 48, fake_i8(11), 16, fake_i32(12), 16}};
    plan_exact("8-bit: ragged, empty, misaligned", ragged, bytes_fn, plan_fn, true);
    std::vector<lb_i8_problem> bad = grid;
    bad[10].lda = bad[10].K - 1;
    plan_exact("8-bit: bad lda", bad, bytes_fn, plan_fn, false);
    bad = grid;
    bad[10].C = nullptr;
    plan_exact("8-bit: null C", bad, bytes_fn, plan_fn, false);
    bad = grid;
    bad[3].K = kBig;
    plan_exact("8-bit: depth overflow", bad, bytes_fn, plan_fn, false);
    EXPECT(gemm_i8_grouped_table_bytes(-1, nullptr) == 0);
    EXPECT(gemm_i8_grouped(0, nullptr, 0, nullptr) == LB_OK);
}

static void calibration_arguments()
{
    EXPECT(lb_calib_sink_bytes() > 0 && lb_calib_clocks_bytes() > 0);
    EXPECT(lb_calib_valu_lane_instr(1, 1000, 8) > 0);
    EXPECT(lb_calib_valu_lane_instr(99, 1000, 8) == 0);
    EXPECT(lb_calib_valu_lane_instr(1, -5, 8) == 0);
    EXPECT(lb_calib_valu_lane_instr(1, 1000, 0) == 0);
    EXPECT(lb_calib_valu_lane_instr(1, kBig, 8) == 0);  // beyond the iteration limit of lb_calib_valu
    EXPECT(lb_calib_valu(1, 1000, 8, nullptr, nullptr, nullptr) == LB_EINVAL);
    EXPECT(lb_calib_valu(99, 1000, 8, fake_i32(1), fake_i32(2), nullptr) == LB_EINVAL);
    EXPECT(lb_calib_stream(7, fake_i8(1), fake_i8(2), 1 << 20, 256, fake_i32(1), nullptr) == LB_EINVAL);
    EXPECT(lb_calib_stream(0, fake_i8(1), fake_i8(2), -16, 256, fake_i32(1), nullptr) == LB_EINVAL);
}

// Shows that the instrumentation is live: a caller that hands the planning call a block 16 bytes shorter than it
// claims must end in a sanitizer report (the library trusts table_bytes, as documented).
static int lie_about_the_table_size()
{
    std::vector<lb_gemm_problem> ps = {{72, 24, 128, fake_u64(1), fake_u64(2), fake_i32(3), 24}};
    const size_t bytes = gemm_grouped_table_bytes(1, 1, ps.data());
    unsigned char *table = static_cast<unsigned char *>(std::malloc(bytes - 16));
    int64_t wg = 0;
    gemm_grouped_plan(1, 1, ps.data(), table, bytes, &wg);
    std::printf("the short block went unnoticed\n");
    std::free(table);
    return 0;
}

int main(int argc, char **argv)
{
    if (argc > 1 && std::strcmp(argv[1], "--lie") == 0)
        return lie_about_the_table_size();
    std::printf("size helpers\n");
    size_helpers();
    std::printf("architecture names\n");
    arch_names();
    std::printf("argument validation of the single calls\n");
    single_call_validation();
    std::printf("dispatch descriptions\n");
    describe_plans();
    std::printf("grouped launch planning (popcount kernels)\n");
    grouped_popcount();
    std::printf("grouped launch planning (8-bit comparator)\n");
    grouped_i8();
    std::printf("calibration arguments\n");
    calibration_arguments();
    std::printf(g_failures ? "%d expectation(s) failed\n" : "all expectations hold (%d failures)\n", g_failures);
    return g_failures ? 1 : 0;
}
