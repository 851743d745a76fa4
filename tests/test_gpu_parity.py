"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by element (bit-exact).

Every test prints what it is about to run (shape, seed, entry point) and flushes, so a failing run names its case.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import bitref, oracle
from paper_2205_09120_amd import binding as lb
from paper_2205_09120_amd import synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lb.lib()  # fail loudly if the HIP library is missing
    yield
    for op in ("bnn", "tnn", "tbn"):
        lb.lb_set_variant(op, -1)


def dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(x).cuda()


def words(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def run_gemm(kind, A, B, C=None, ldc=None):
    M, K = A.shape
    N = B.shape[1]
    dA, dB = dev(A), dev(B)
    Ap, Bp = lb.pack_a(kind, dA), lb.pack_b(kind, dB)
    out = lb.gemm(kind, M, N, K, Ap, Bp, C, ldc)
    torch.cuda.synchronize()
    return out


# ------------------------------------------------------------------------------------------------ packing

PACK_SHAPES = [(1, 1), (3, 63), (5, 64), (7, 65), (64, 576), (130, 1000), (257, 129), (33, 4096 + 17)]


@pytest.mark.parametrize("rows,K", PACK_SHAPES)
@pytest.mark.parametrize("ternary", [True, False])
def test_pack_depth_contiguous(rows, K, ternary):
    say(f"pack depth-contiguous rows={rows} K={K} ternary={ternary}")
    X, _ = synth.make_custom("tnn" if ternary else "bnn", rows, 1, K, seed=rows * 7 + K)
    for lda in (K, ((K + 15) // 16) * 16, ((K + 15) // 16) * 16 + 16):
        buf = np.zeros((rows, lda), dtype=np.int8)
        buf[:, :K] = X
        d = dev(buf)
        f = lb.pack_ternary if ternary else lb.pack_binary
        got = words(f(d, rows, K, lda, 1))
        torch.cuda.synchronize()
        want = (bitref.pack_ternary(X) if ternary else bitref.pack_binary(X)).reshape(-1)
        assert np.array_equal(got, want), f"lda={lda}"


@pytest.mark.parametrize("rows,K", PACK_SHAPES + [(784, 2304), (8, 300)])
@pytest.mark.parametrize("ternary", [True, False])
def test_pack_depth_strided(rows, K, ternary):
    say(f"pack depth-strided rows={rows} K={K} ternary={ternary}")
    _, B = synth.make_custom("tnn" if ternary else "bnn", 1, rows, K, seed=rows * 3 + K)   # K x rows
    for ldb in (rows, ((rows + 3) // 4) * 4, ((rows + 3) // 4) * 4 + 8):
        buf = np.zeros((K, ldb), dtype=np.int8)
        buf[:, :rows] = B
        d = dev(buf)
        f = lb.pack_ternary if ternary else lb.pack_binary
        got = words(f(d, rows, K, 1, ldb))
        torch.cuda.synchronize()
        Xt = np.ascontiguousarray(B.T)
        want = (bitref.pack_ternary(Xt) if ternary else bitref.pack_binary(Xt)).reshape(-1)
        assert np.array_equal(got, want), f"ldb={ldb}"


def test_pack_misaligned_source_and_illegal_values():
    say("pack misaligned source / values outside the legal sets")
    rng = np.random.default_rng(5)
    X = rng.integers(-128, 128, size=(9, 200), dtype=np.int8)         # any int8: encoded by sign
    big = np.zeros(9 * 200 + 3, dtype=np.int8)
    big[3:] = X.reshape(-1)
    d = dev(big)[3:]                                                  # data pointer off by 3 bytes
    got_t = words(lb.pack_ternary(d, 9, 200, 200, 1))
    got_b = words(lb.pack_binary(d, 9, 200, 200, 1))
    torch.cuda.synchronize()
    assert np.array_equal(got_t, bitref.pack_ternary(X).reshape(-1))
    assert np.array_equal(got_b, bitref.pack_binary(X).reshape(-1))
    dX = dev(X)
    assert np.array_equal(words(lb.pack_ternary(dX, 9, 200, 200, 1)), bitref.pack_ternary(X).reshape(-1))
    Xt = np.ascontiguousarray(X.T)                                    # 200 x 9 viewed as depth-strided (rows=9... )
    dXt = dev(Xt)
    got = words(lb.pack_ternary(dXt, 9, 200, 1, 9))
    torch.cuda.synchronize()
    assert np.array_equal(got, bitref.pack_ternary(X).reshape(-1))
    planes = got.reshape(-1, 2)
    assert not np.any(planes[:, 0] & planes[:, 1])                    # never the invalid code (1,1)


# ------------------------------------------------------------------------------------------------ GEMM, benchmark configs

@pytest.mark.parametrize("name", ["cfg1_tnn_conv3x3x64_16x16", "cfg2_bnn_conv3x3x128_56x56",
                                  "cfg3_tbn_conv3x3x256_28x28", "cfg5_tnn_fc_n8", "cfg5_tbn_fc_n8",
                                  "cfg5_bnn_fc_n8"])
def test_gemm_configs_full(name):
    w = synth.WORKLOADS[name]
    say(f"gemm_{w.kind} {name} M={w.M} N={w.N} K={w.K} seed={w.seed}")
    A, B = synth.make_inputs(w)
    got = run_gemm(w.kind, A, B).cpu().numpy()
    want = oracle.gemm(A, B)
    assert np.array_equal(got, want)


def test_gemm_headline_full_size():
    """cfg4 at full size in the default launch configuration (the one bench.py times): every element."""
    w = synth.WORKLOADS[synth.HEADLINE]
    say(f"gemm_tnn {w.name} M={w.M} N={w.N} K={w.K} seed={w.seed} (full oracle)")
    A, B = synth.make_inputs(w)
    got = run_gemm("tnn", A, B).cpu().numpy()
    say("  gpu done; running oracle")
    want = oracle.gemm(A, B)
    assert np.array_equal(got, want)
    n11_bound = ((A != 0).sum(axis=1, dtype=np.int64)[:, None])       # |c| <= nnz(row) is implied by |c| <= n11
    assert np.all(np.abs(got) <= n11_bound)


# ------------------------------------------------------------------------------------------------ GEMM, edge shapes, all variants

EDGE_SHAPES = [(70, 70, 40 * 64 + 1), (1, 1, 1), (1, 1, 64), (1, 70, 65), (70, 1, 63), (5, 7, 130), (33, 65, 64), (64, 64, 128),
               (65, 129, 200), (100, 300, 577), (8, 520, 1000), (130, 8, 2000), (257, 513, 320)]


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_edge_shapes_all_variants(kind):
    nvar = lb.lb_num_variants(kind)
    try:
        for v in list(range(nvar)) + [-1]:
            lb.lb_set_variant(kind, v)
            for (M, N, K) in EDGE_SHAPES:
                say(f"gemm_{kind} variant={v} ({lb.lb_variant_name(kind, v)}) M={M} N={N} K={K}")
                A, B = synth.make_custom(kind, M, N, K, seed=M + 3 * N + 7 * K)
                got = run_gemm(kind, A, B).cpu().numpy()
                assert np.array_equal(got, oracle.gemm(A, B)), (v, M, N, K)
    finally:
        lb.lb_set_variant(kind, -1)


SKINNY_SHAPES = [(64, 1, 64), (64, 8, 1), (100, 9, 16384 + 70), (4096, 16, 300), (1000, 3, 20000), (3, 1000, 700),
                 (16, 64, 16385), (8, 4100, 130), (257, 8, 16384), (5000, 7, 65),
                 # deep enough for the depth-split kernel (depth >= 2048 and not many more rows than depth) ...
                 (300, 8, 2048 + 70), (4096, 16, 4100), (2100, 5, 2049), (5, 3000, 4000), (9, 2500, 2304),
                 (20000, 2, 16384 + 64), (7000, 11, 9000),
                 # 9..32 short strings: 16 or 32 of them per workgroup, the long operand still streamed once
                 (1000, 12, 5000), (2000, 16, 4096), (1000, 24, 8192 + 70), (2048, 32, 16384), (900, 17, 4100),
                 (20, 3000, 16384), (32, 1030, 9000),
                 # ... and narrow shapes that the tiled kernel serves: many shallow rows, 1 / 8 / 16 strings
                 (30000, 1, 600), (30000, 8, 1000), (30000, 13, 2500), (20000, 16, 20000 // 8), (12, 30000, 1000)]


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_skinny_shapes(kind):
    """Shapes with one narrow side: the depth-split kernel (both orientations, several depth chunks, tails) where
    the depth is large against the row count, the tiled kernel with low tiles elsewhere."""
    for (M, N, K) in SKINNY_SHAPES:
        say(f"gemm_{kind} skinny M={M} N={N} K={K}")
        A, B = synth.make_custom(kind, M, N, K, seed=M + 5 * N + 11 * K)
        got = run_gemm(kind, A, B).cpu().numpy()
        assert np.array_equal(got, oracle.gemm(A, B)), (M, N, K)


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_skinny_every_configuration(kind):
    """Every (rows per wave, waves per workgroup) configuration of the depth-split kernel, for 8, 16 and 32 short
    strings per workgroup and both operand roles; forcing a configuration also forces that kernel."""
    shapes = [(300, 5, 700), (130, 13, 1000), (70, 29, 600), (7, 200, 900), (31, 150, 1300), (257, 32, 2048 + 64)]
    try:
        for cfg in range(lb.lb_num_variants(3)):
            lb.lb_set_variant(3, cfg)
            for (M, N, K) in shapes:
                say(f"gemm_{kind} skinny configuration {cfg} M={M} N={N} K={K}")
                assert "depth-split-across-lanes" in lb.lb_describe_plan(kind, M, N, K)
                A, B = synth.make_custom(kind, M, N, K, seed=cfg * 100 + M + N)
                ldc = N + 2
                C = torch.full((M, ldc), -5, dtype=torch.int32, device="cuda")
                run_gemm(kind, A, B, C=C, ldc=ldc)
                got = C.cpu().numpy()
                assert np.array_equal(got[:, :N], oracle.gemm(A, B)), (cfg, M, N, K)
                assert np.all(got[:, N:] == -5)
    finally:
        lb.lb_set_variant(3, -1)


STREAM_SHAPES = [(9000, 8, 4096), (10000, 5, 8192), (5000, 8, 16384 + 128), (70000, 8, 2048), (33000, 3, 24576),
                 (8, 9000, 4096), (3, 40000, 8192), (4100, 7, 64 * 77), (1, 8, 16384), (4097, 1, 32768),
                 (600, 8, 65536), (2, 5000, 16384 + 70)]


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_skinny_streaming_kernel(kind):
    """The streaming depth-split kernel (short strings resident in LDS, waves walking over row groups with a ring of
    loads in flight): one and two rows per wave, ring depths 1 / 2 / 4, depths that are and are not multiples of a
    wave-wide step, more row groups than waves, both operand roles, odd word counts (binary strings then take the
    chunked kernel), a padded ldc."""
    try:
        for cfg in (8, 9, -1):
            lb.lb_set_variant(3, cfg)
            for (M, N, K) in STREAM_SHAPES:
                say(f"gemm_{kind} streaming skinny configuration {cfg} M={M} N={N} K={K}")
                A, B = synth.make_custom(kind, M, N, K, seed=cfg * 10 + M + N + K)
                ldc = N + 1
                C = torch.full((M, ldc), -9, dtype=torch.int32, device="cuda")
                run_gemm(kind, A, B, C=C, ldc=ldc)
                got = C.cpu().numpy()
                assert np.array_equal(got[:, :N], oracle.gemm(A, B)), (cfg, M, N, K)
                assert np.all(got[:, N:] == -9)
    finally:
        lb.lb_set_variant(3, -1)


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_depth_split(kind):
    """Few tiles and a long depth: the depth is split over workgroups whose partial products are added into a cleared
    C (int32 atomics).  Depths that are not multiples of 64 (eq. (6) needs the true depth of every range), ragged
    tiles, a padded ldc whose padding must stay untouched, and a C that holds garbage before the call."""
    for (M, N, K) in [(64, 64, 8192 + 70), (100, 200, 12001), (130, 257, 30000), (24, 700, 9000), (1, 64, 8192),
                      (17, 65, 65536 + 1), (256, 256, 8192),
                      # lanes own rows of C (narrow N; gemm_tbn in general): the partial results go through LDS
                      (512, 49, 16384 + 70), (1000, 40, 20001), (70, 33, 12000), (257, 63, 10240)]:
        ldc = N + 3
        say(f"gemm_{kind} depth-split M={M} N={N} K={K} ldc={ldc}")
        A, B = synth.make_custom(kind, M, N, K, seed=M + 3 * N + K)
        C = torch.full((M, ldc), 12345, dtype=torch.int32, device="cuda")
        run_gemm(kind, A, B, C=C, ldc=ldc)
        got = C.cpu().numpy()
        assert np.array_equal(got[:, :N], oracle.gemm(A, B)), (M, N, K)
        assert np.all(got[:, N:] == 12345)


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_paper_shape_grid(kind):
    """All 64 height x width x depth shapes of the paper's timing experiment (Section IV-B)."""
    for idx, (H, W, D) in enumerate(synth.paper_shape_grid()):
        if idx % 8 == 0:
            say(f"gemm_{kind} paper grid shapes {idx}..{idx + 7}: first {H}x{W}x{D}")
        A, B = synth.make_custom(kind, H, W, D, seed=1000 + idx)
        got = run_gemm(kind, A, B).cpu().numpy()
        assert np.array_equal(got, oracle.gemm(A, B)), (H, W, D)


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_ldc_and_untouched_padding(kind):
    M, N, K, ldc = 37, 50, 333, 64
    say(f"gemm_{kind} ldc M={M} N={N} K={K} ldc={ldc}")
    A, B = synth.make_custom(kind, M, N, K, seed=99)
    C = torch.full((M, ldc), -777, dtype=torch.int32, device="cuda")
    run_gemm(kind, A, B, C=C, ldc=ldc)
    got = C.cpu().numpy()
    assert np.array_equal(got[:, :N], oracle.gemm(A, B))
    assert np.all(got[:, N:] == -777)


EIGHT_WAVE_SHAPES = [  # (M, N, K, part of the plan the shape-based dispatch must name)
    ("tnn", 515, 8200, 2304, "ts4 tv2 w8 kg8 sg4"),    # ragged rows and columns, 17 x 65 tiles of 32 x 128
    ("tnn", 1000, 4100, 2100, "ts4 tv2 w8 kg8 sg4"),   # depth not a multiple of 64
    ("tnn", 1000, 3100, 2400, "ts4 tv1 w8 kg16 sg4"),  # fewer than 1024 wide tiles: the 32 x 64 tile of eight waves
    ("bnn", 515, 8200, 2304, "ts4 tv2 w8 kg8 sg4"),
    ("bnn", 512, 4096, 2112, "ts4 tv2 w8 kg8 sg4"),    # exactly two workgroups per compute unit
    ("tbn", 2060, 4100, 2100, "ts8 tv2 w8 kg8 sg4"),   # lanes own rows of C: results leave through LDS, written through
    ("tbn", 515, 8200, 2304, "ts8 tv1 w4 kg8 sg4"),
    ("tnn", 70000, 13, 300, "B on the scalar side"),   # narrow N: same store path from the 16-row tile
]


@pytest.mark.parametrize("kind,M,N,K,plan", EIGHT_WAVE_SHAPES)
def test_gemm_eight_wave_tiles_and_row_wise_stores(kind, M, N, K, plan):
    """The instances the dispatch takes for a thousand tiles and more, at ragged extents, with ldc > N."""
    got_plan = lb.lb_describe_plan(kind, M, N, K)
    say(f"gemm_{kind} M={M} N={N} K={K}: {got_plan}")
    assert plan in got_plan
    A, B = synth.make_custom(kind, M, N, K, seed=M + N + K)
    ldc = N + 5
    C = torch.full((M, ldc), -777, dtype=torch.int32, device="cuda")
    run_gemm(kind, A, B, C=C, ldc=ldc)
    got = C.cpu().numpy()
    assert np.array_equal(got[:, :N], oracle.gemm(A, B))
    assert np.all(got[:, N:] == -777)


def test_same_no_zero_matrix_through_all_three_entry_points():
    """A ternary matrix without zeros is also a binary matrix: the three entry points must agree on it."""
    say("cross-check tnn/tbn/bnn on +-1 matrices")
    A, B = synth.make_custom("bnn", 77, 91, 450, seed=12)
    want = oracle.gemm(A, B)
    for kind in ("bnn", "tnn", "tbn"):
        assert np.array_equal(run_gemm(kind, A, B).cpu().numpy(), want), kind


def test_special_cases_on_gpu():
    say("special cases: zero matrix, all ones, negation")
    A, B = synth.make_custom("tnn", 40, 70, 260, seed=21)
    assert not run_gemm("tnn", np.zeros_like(A), B).cpu().numpy().any()
    ones = np.ones_like(A)
    assert np.array_equal(run_gemm("tnn", ones, B).cpu().numpy(),
                          np.broadcast_to(B.sum(axis=0, dtype=np.int32), (40, 70)))
    assert np.array_equal(run_gemm("tnn", -A, B).cpu().numpy(), -oracle.gemm(A, B))


def test_deterministic():
    w = synth.WORKLOADS["cfg3_tbn_conv3x3x256_28x28"]
    say("determinism", w.name)
    A, B = synth.make_inputs(w)
    a = run_gemm(w.kind, A, B).cpu().numpy()
    b = run_gemm(w.kind, A, B).cpu().numpy()
    assert np.array_equal(a, b)


# ------------------------------------------------------------------------------------------------ 16-bit C (Section III)

@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_c16_matches_oracle(kind):
    """Signed 16-bit C: same integers as the oracle (|c| <= K <= 32767), on the tiled kernel in both orientations,
    every tile variant, the skinny kernel, a padded ldc (padding untouched) and an odd C address."""
    shapes = [(64, 256, 576), (130, 70, 100), (257, 300, 1000), (70, 40, 32767), (300, 8, 700), (9, 400, 260),
              (512, 70, 64), (1, 1, 1), (33, 129, 65)]
    for (M, N, K) in shapes:
        A, B = synth.make_custom(kind, M, N, K, seed=M * 11 + N * 7 + K)
        want = oracle.gemm(A, B)
        assert np.abs(want).max() <= 32767
        Ap, Bp = lb.pack_a(kind, dev(A)), lb.pack_b(kind, dev(B))
        try:
            for v in [-1] + list(range(lb.lb_num_variants(kind))):
                lb.lb_set_variant(kind, v)
                ldc = N + 3
                say(f"gemm_c16 {kind} M={M} N={N} K={K} variant={v} ldc={ldc}")
                flat = torch.full((M * ldc + 1,), 12345, dtype=torch.int16, device="cuda")
                C = flat[1:].view(M, ldc)                             # 2-byte aligned only
                lb.gemm_c16(kind, M, N, K, Ap, Bp, C, ldc)
                torch.cuda.synchronize()
                got = C.cpu().numpy()
                assert got.dtype == np.int16
                assert np.array_equal(got[:, :N].astype(np.int32), want), (M, N, K, v)
                assert np.all(got[:, N:] == 12345) and int(flat[0]) == 12345
        finally:
            lb.lb_set_variant(kind, -1)


def test_gemm_c16_extreme_values_and_depth_limit():
    """K = 32767 with operands that reach +K and -K; K = 32768 is refused."""
    K = 32767
    A = np.ones((5, K), dtype=np.int8)
    B = np.ones((K, 70), dtype=np.int8)
    B[:, 1::2] = -1
    say("gemm_c16 extremes")
    for kind in ("bnn", "tnn", "tbn"):
        got = lb.gemm_c16(kind, 5, 70, K, lb.pack_a(kind, dev(A)), lb.pack_b(kind, dev(B))).cpu().numpy()
        assert np.all(got[:, 0::2] == K) and np.all(got[:, 1::2] == -K)
    with pytest.raises(lb.LowbitError) as e:
        lb.gemm_c16("bnn", 5, 70, K + 1, lb.pack_a("bnn", dev(A)), lb.pack_b("bnn", dev(B)))
    assert e.value.status == lb.LB_EOVERFLOW


# ------------------------------------------------------------------------------------------------ int8 matrix-core comparator

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (64, 256, 576), (130, 70, 100), (128, 128, 64), (257, 300, 1000),
                                   (512, 784, 2304), (33, 8, 4096), (300, 515, 131), (256, 256, 64),
                                   (4096, 8, 2048), (100, 5, 3000), (64, 16, 4100), (257, 9, 16), (1000, 8, 8192),
                                   (256, 128, 64), (512, 256, 128), (256, 384, 192), (512, 128, 448), (300, 516, 144),
                                   (20, 24, 16), (700, 260, 1040), (256, 256, 128), (512, 512, 384),
                                   (256, 768, 1280), (768, 256, 256), (257, 304, 256), (100, 48, 192),
                                   (130, 1040, 384), (513, 3088, 256), (65, 16, 64), (1, 32, 128)])
def test_i8_mfma(M, N, K):
    say(f"gemm_i8_mfma M={M} N={N} K={K}")
    rng = np.random.default_rng(M + N + K)
    A = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
    B = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    want = oracle.gemm(A, B)
    try:
        for tile in range(-1, lb.lb_num_variants(4)):  # 4-wave tiles and the wave-specialised instances
            lb.lb_set_variant(4, tile)
            got = lb.gemm_i8_mfma(M, N, K, dev(A), K, dev(B), N)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), want), tile
    finally:
        lb.lb_set_variant(4, -1)


@pytest.mark.parametrize("M,N,K", [(2048, 16384, 192), (2048, 16512, 208), (2300, 16384, 64), (2048, 16384, 384),
                                   (1100, 4112, 256), (640, 6416, 128), (2048, 2064, 384)])
def test_i8_and_u8_large_default_path(M, N, K):
    """Shapes large enough for the shape-based choice to take the direct-to-LDS kernel (whole tiles, depth a multiple
    of 128) or the wave-specialised one (everything else, ragged tiles included)."""
    say(f"gemm_i8_mfma / gemm_u8_mfma default path M={M} N={N} K={K}")
    rng = np.random.default_rng(M + N + K)
    A = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
    B = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    got = lb.gemm_i8_mfma(M, N, K, dev(A), K, dev(B), N)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.gemm(A, B))
    Au, Bu = A.view(np.uint8), B.view(np.uint8)
    got = lb.gemm_u8_mfma(M, N, K, dev(Au), K, dev(Bu), N, 3, 250)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.gemm_u8_zero_point(Au, Bu, 3, 250))


def test_i8_u8_random_shapes_and_leading_dimensions():
    """40 seeded draws through the shape-based dispatch of the 8-bit comparator: extents log-uniform, N and K often
    multiples of 16 / 64 (the direct-to-LDS instances) and often not (the others), padded leading dimensions, C
    padding must stay untouched."""
    rng = np.random.default_rng(77)
    for it in range(40):
        M = int(np.exp(rng.uniform(0, np.log(900))))
        N = int(np.exp(rng.uniform(0, np.log(1500))))
        K = int(np.exp(rng.uniform(0, np.log(3000))))
        if rng.random() < 0.6:
            N = max(16, N // 16 * 16)
        if rng.random() < 0.7:
            K = max(64, K // 64 * 64)
        lda = K + int(rng.choice([0, 16, 48, 5]))
        ldb = N + int(rng.choice([0, 16, 64, 3]))
        ldc = N + int(rng.choice([0, 4, 7]))
        zA, zB = int(rng.integers(0, 256)), int(rng.integers(0, 256))
        say(f"8-bit random {it}: M={M} N={N} K={K} lda={lda} ldb={ldb} ldc={ldc} zA={zA} zB={zB}")
        A = np.zeros((M, lda), dtype=np.int8)
        B = np.zeros((K, ldb), dtype=np.int8)
        A[:, :K] = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
        B[:, :N] = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
        A[:, K:] = 77                                                     # padding must never reach a product
        B[:, N:] = -55
        C = torch.full((M, ldc), 4242, dtype=torch.int32, device="cuda")
        lb.gemm_i8_mfma(M, N, K, dev(A), lda, dev(B), ldb, C, ldc)
        torch.cuda.synchronize()
        got = C.cpu().numpy()
        assert np.array_equal(got[:, :N], oracle.gemm(np.ascontiguousarray(A[:, :K]), np.ascontiguousarray(B[:, :N])))
        assert np.all(got[:, N:] == 4242)
        Au, Bu = A.view(np.uint8), B.view(np.uint8)
        C.fill_(4242)
        lb.gemm_u8_mfma(M, N, K, dev(Au), lda, dev(Bu), ldb, zA, zB, C, ldc)
        torch.cuda.synchronize()
        got = C.cpu().numpy()
        want = oracle.gemm_u8_zero_point(np.ascontiguousarray(Au[:, :K]), np.ascontiguousarray(Bu[:, :N]), zA, zB)
        assert np.array_equal(got[:, :N], want)
        assert np.all(got[:, N:] == 4242)


def test_i8_mfma_on_ternary_config():
    w = synth.WORKLOADS["cfg1_tnn_conv3x3x64_16x16"]
    say("gemm_i8_mfma", w.name)
    A, B = synth.make_inputs(w)
    got = lb.gemm_i8_mfma(w.M, w.N, w.K, dev(A), w.K, dev(B), w.N)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.gemm(A, B))


# ------------------------------------------------------------------------------------------------ streams, ldc on every path, random shapes

def test_non_default_stream_and_overlap():
    """Calls enqueue on the stream they are given: two problems on two streams, results checked after one sync."""
    say("two streams")
    A1, B1 = synth.make_custom("tnn", 300, 500, 900, seed=31)
    A2, B2 = synth.make_custom("bnn", 200, 700, 1300, seed=32)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    dA1, dB1, dA2, dB2 = dev(A1), dev(B1), dev(A2), dev(B2)
    torch.cuda.synchronize()
    with torch.cuda.stream(s1):
        C1 = lb.gemm("tnn", 300, 500, 900, lb.pack_a("tnn", dA1), lb.pack_b("tnn", dB1))
    with torch.cuda.stream(s2):
        C2 = lb.gemm("bnn", 200, 700, 1300, lb.pack_a("bnn", dA2, stream=s2), lb.pack_b("bnn", dB2, stream=s2),
                     stream=s2)
    torch.cuda.synchronize()
    assert np.array_equal(C1.cpu().numpy(), oracle.gemm(A1, B1))
    assert np.array_equal(C2.cpu().numpy(), oracle.gemm(A2, B2))


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
@pytest.mark.parametrize("shape", [(300, 8, 700), (9, 400, 260), (512, 70, 64)])
def test_ldc_on_skinny_and_transposed_paths(kind, shape):
    M, N, K = shape
    ldc = N + 5
    say(f"gemm_{kind} ldc={ldc} M={M} N={N} K={K}")
    A, B = synth.make_custom(kind, M, N, K, seed=M + N + K)
    C = torch.full((M, ldc), 12345, dtype=torch.int32, device="cuda")
    run_gemm(kind, A, B, C=C, ldc=ldc)
    got = C.cpu().numpy()
    assert np.array_equal(got[:, :N], oracle.gemm(A, B))
    assert np.all(got[:, N:] == 12345)


def test_random_shapes():
    """60 seeded random (kind, M, N, K) draws, log-uniform extents, through the shape-based dispatch."""
    rng = np.random.default_rng(2024)
    for it in range(60):
        kind = ("bnn", "tnn", "tbn")[int(rng.integers(0, 3))]
        M, N = (int(np.exp(rng.uniform(0, np.log(700)))) for _ in range(2))
        K = int(np.exp(rng.uniform(0, np.log(5000))))
        say(f"random shape {it}: gemm_{kind} M={M} N={N} K={K}")
        A, B = synth.make_custom(kind, M, N, K, seed=5000 + it)
        assert np.array_equal(run_gemm(kind, A, B).cpu().numpy(), oracle.gemm(A, B)), (kind, M, N, K)


def test_sparse_and_dense_ternary_extremes():
    """Ternary operands with P(0) = 0 and P(0) = 0.98 (and the all-zero operand on one side)."""
    say("ternary density extremes")
    for p0 in (0.0, 0.98):
        A, B = synth.make_custom("tnn", 130, 260, 777, seed=int(p0 * 100) + 1, p0=p0)
        assert np.array_equal(run_gemm("tnn", A, B).cpu().numpy(), oracle.gemm(A, B))
        A, B = synth.make_custom("tbn", 130, 260, 777, seed=int(p0 * 100) + 2, p0=p0)
        assert np.array_equal(run_gemm("tbn", A, B).cpu().numpy(), oracle.gemm(A, B))
    A, B = synth.make_custom("tbn", 70, 90, 300, seed=3)
    assert not run_gemm("tbn", np.zeros_like(A), B).cpu().numpy().any()


# ------------------------------------------------------------------------------------------------ U8 with zero points (eq. (3))

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (64, 256, 576), (130, 70, 100), (257, 300, 1000), (512, 784, 2304),
                                   (33, 8, 4096), (300, 515, 131), (1024, 2048, 320), (257, 304, 256), (100, 48, 192),
                                   (513, 3088, 384), (1100, 4112, 128)])
def test_u8_zero_point_gemm(M, N, K):
    rng = np.random.default_rng(M * 3 + N * 5 + K)
    A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    B = rng.integers(0, 256, size=(K, N), dtype=np.uint8)
    for zA, zB in ((0, 0), (128, 128), (17, 240)):
        say(f"gemm_u8_mfma M={M} N={N} K={K} zA={zA} zB={zB}")
        got = lb.gemm_u8_mfma(M, N, K, dev(A), K, dev(B), N, zA, zB)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.gemm_u8_zero_point(A, B, zA, zB)), (zA, zB)


def test_u8_extreme_values_and_depth_limit():
    say("gemm_u8_mfma extremes")
    K = 33025
    A = np.full((70, K), 255, dtype=np.uint8)
    B = np.zeros((K, 66), dtype=np.uint8)
    got = lb.gemm_u8_mfma(70, 66, K, dev(A), K, dev(B), 66, 0, 255)
    torch.cuda.synchronize()
    assert np.all(got.cpu().numpy() == -K * 255 * 255)
    with pytest.raises(lb.LowbitError) as e:
        lb.gemm_u8_mfma(70, 66, K + 1, dev(A), K + 1, dev(B), 66, 0, 255)
    assert e.value.status == lb.LB_EOVERFLOW


# ------------------------------------------------------------------------------------------------ calibration kernels

def test_calibration_kernels_run_and_copy_is_exact():
    say("calibration kernels")
    sink = torch.zeros(lb.lb_calib_sink_bytes() // 4, dtype=torch.int32, device="cuda")
    clk = torch.zeros(lb.lb_calib_clocks_bytes() // 8, dtype=torch.int64, device="cuda")
    iters, seed = 8, 0x9e3779b9
    # what every thread of the binary and the popcount-only chain must have counted: 8 chains, a[c] = seed*(c+1) + thread,
    # s[c] = (seed >> c) ^ (workgroup * (c+3)), in 32-bit arithmetic
    blk = np.arange(2048, dtype=np.uint64)[:, None, None]
    tid = np.arange(256, dtype=np.uint64)[None, :, None]
    c = np.arange(8, dtype=np.uint64)[None, None, :]
    a = (seed * (c + 1) + tid) & 0xffffffff
    sc = ((seed >> c) ^ (blk * (c + 3))) & 0xffffffff
    popc = lambda x: np.array([bin(int(v)).count("1") for v in x.ravel()]).reshape(x.shape)
    want_bcnt = np.broadcast_to(popc(a).sum(axis=2) * iters, (2048, 256))
    for waves in (8, 3):
        nthreads = 256 * waves * 256
        sink.zero_()
        lb.lb_calib_valu(6, iters, sink, clk, waves)
        torch.cuda.synchronize()
        assert np.array_equal(sink.cpu().numpy()[:nthreads].reshape(-1, 256), want_bcnt[: 256 * waves])
        assert not sink.cpu().numpy()[nthreads:].any()
        ck = clk.cpu().numpy().reshape(-1, 2)[: 256 * waves]
        assert (ck > 0).all()                                   # both counters advanced in every workgroup
    lb.lb_calib_valu(0, iters, sink, None, 1)
    torch.cuda.synchronize()
    x = a[:, :, :] ^ sc[:256]
    want = np.array([[sum(bin(int(v)).count("1") for v in x[b, t]) for t in range(256)] for b in range(4)]) * iters
    assert np.array_equal(sink.cpu().numpy()[: 4 * 256].reshape(4, 256), want)
    for mix in (1, 2, 3, 4, 5):
        lb.lb_calib_valu(mix, iters, sink, clk)
    torch.cuda.synchronize()
    assert lb.lb_calib_valu_lane_instr(1, iters, 8) == 2048 * 256 * iters * 32
    n = 1 << 20
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    lb.lb_calib_stream(2, src, dst, n, sink)
    lb.lb_calib_stream(0, src, None, n, sink)
    lb.lb_calib_stream(0, src, None, n, sink, 256)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    lb.lb_calib_stream(1, None, dst, n, sink)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy().view(np.uint32)[:8], np.array([1, 2, 3, 4, 1, 2, 3, 4], dtype=np.uint32))
