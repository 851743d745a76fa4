"""GPU parity of the matrix-core product on 4-bit floats (pack_t4 + gemm_t4_mfma): packed bytes bit for bit against the
reference packer, products bit for bit against the oracle (the definition C = A B), for ternary, ternary-binary and
binary operands."""
import numpy as np
import pytest
import torch

from oracle import oracle, t4ref
from paper_2205_09120_amd import binding as lb
from paper_2205_09120_amd import synth

pytestmark = pytest.mark.gpu


def _pack_both(A, B):
    M, K = A.shape
    N = B.shape[1]
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    return lb.pack_t4(dA, M, K, K, 1), lb.pack_t4(dB, N, K, 1, N)


@pytest.mark.parametrize("rows,K", [(1, 1), (5, 63), (32, 128), (33, 129), (70, 300), (257, 1000)])
def test_pack_t4_matches_reference_packer(rows, K):
    rng = np.random.default_rng(rows * 7 + K)
    X = rng.integers(-1, 2, size=(rows, K)).astype(np.int8)
    want = t4ref.pack_t4(X)
    got = lb.pack_t4(torch.from_numpy(X).cuda(), rows, K, K, 1)
    assert np.array_equal(got.cpu().numpy(), want)
    XT = np.ascontiguousarray(X.T)                  # the same matrix handed over depth-strided
    got = lb.pack_t4(torch.from_numpy(XT).cuda(), rows, K, 1, rows)
    assert np.array_equal(got.cpu().numpy(), want)


def test_pack_t4_takes_values_by_sign_and_honours_leading_dimensions():
    rng = np.random.default_rng(5)
    rows, K, ld = 45, 200, 211
    buf = rng.integers(-128, 128, size=(rows, ld)).astype(np.int8)
    want = t4ref.pack_t4(buf[:, :K])
    got = lb.pack_t4(torch.from_numpy(buf).cuda(), rows, K, ld, 1)
    assert np.array_equal(got.cpu().numpy(), want)
    bufT = np.zeros((K, rows + 3), dtype=np.int8)
    bufT[:, :rows] = buf[:, :K].T
    got = lb.pack_t4(torch.from_numpy(bufT).cuda(), rows, K, 1, rows + 3)
    assert np.array_equal(got.cpu().numpy(), want)


# the last one has a partial last round of 256 x 256 tiles (289 tiles): two launches, the second with small tiles
SHAPES = [(1, 1, 1), (3, 5, 7), (64, 64, 128), (65, 33, 129), (100, 260, 300), (256, 256, 512), (300, 520, 1000),
          (513, 130, 4608), (4100, 4300, 2100)]


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("kind", ["tnn", "tbn", "bnn"])
@pytest.mark.parametrize("inst", [-1, 0, 1, 2, 3])
def test_gemm_t4_matches_oracle(M, N, K, kind, inst):
    A, B = synth.make_custom(kind, M, N, K, seed=M * 31 + N * 7 + K)
    Ap, Bp = _pack_both(A, B)
    lb.lb_set_variant(5, inst)
    try:
        C = lb.gemm_t4_mfma(M, N, K, Ap, Bp)
    finally:
        lb.lb_set_variant(5, -1)
    assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B))


def test_gemm_t4_leading_dimension_of_c():
    M, N, K, ldc = 70, 90, 256, 101
    A, B = synth.make_custom("tnn", M, N, K, seed=11)
    Ap, Bp = _pack_both(A, B)
    C = torch.full((M, ldc), -7, dtype=torch.int32, device="cuda")
    lb.gemm_t4_mfma(M, N, K, Ap, Bp, C, ldc)
    got = C.cpu().numpy()
    assert np.array_equal(got[:, :N], oracle.gemm(A, B))
    assert (got[:, N:] == -7).all()


def test_gemm_t4_extreme_sums_are_exact():
    """All products +1 (and all -1) at a depth of 2^21: the largest magnitudes the accumulation sees stay exact."""
    M, N, K = 40, 50, 1 << 21
    A = np.ones((M, K), dtype=np.int8)
    B = np.ones((K, N), dtype=np.int8)
    B[:, ::2] = -1
    rng = np.random.default_rng(2)
    A[rng.integers(0, M, 300), rng.integers(0, K, 300)] = 0
    Ap, Bp = _pack_both(A, B)
    C = lb.gemm_t4_mfma(M, N, K, Ap, Bp)
    assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B))


def test_gemm_t4_headline_shape_against_the_popcount_kernel_and_the_oracle():
    """cfg4 (1024 x 50176 x 4608, the benchmark's operands) in the launch configuration the benchmark times: every
    output equals gemm_tnn's, and sampled outputs plus a block equal the oracle's."""
    w = synth.WORKLOADS["cfg4_tnn_conv3x3x512_b16_56x56"]
    A, B = synth.make_inputs(w)
    M, N, K = w.M, w.N, w.K
    Ap, Bp = _pack_both(A, B)
    C = lb.gemm_t4_mfma(M, N, K, Ap, Bp)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    C2 = lb.gemm_tnn(M, N, K, lb.pack_a("tnn", dA), lb.pack_b("tnn", dB))
    assert torch.equal(C, C2)
    Ch = C.cpu().numpy()
    rng = np.random.default_rng(44)
    ii, jj = rng.integers(0, M, 4000), rng.integers(0, N, 4000)
    assert np.array_equal(Ch[ii, jj], oracle.gemm_samples(A, B, ii, jj))
    cols = slice(N - 300, N)
    assert np.array_equal(Ch[:64, cols], oracle.gemm(np.ascontiguousarray(A[:64]), np.ascontiguousarray(B[:, cols])))


def test_t4_random_sweep():
    rng = np.random.default_rng(77)
    try:
        for n in range(1, 121):
            r = rng.random()
            if r < 0.25:
                M, N, K = int(rng.integers(1, 40)), int(np.exp(rng.uniform(0, np.log(3000)))), int(np.exp(rng.uniform(0, np.log(20000))))
            elif r < 0.5:
                M, N, K = int(np.exp(rng.uniform(0, np.log(3000)))), int(rng.integers(1, 40)), int(np.exp(rng.uniform(0, np.log(20000))))
            else:
                M, N, K = (int(np.exp(rng.uniform(0, np.log(1200)))) for _ in range(3))
            kind = ("tnn", "tbn", "bnn")[int(rng.integers(0, 3))]
            inst = int(rng.integers(-1, lb.lb_num_variants(5)))
            lda, ldb, ldc = K + int(rng.choice([0, 1, 16, 5])), N + int(rng.choice([0, 1, 4, 7])), N + int(rng.choice([0, 3]))
            print(f"[{n}] t4 {kind} M={M} N={N} K={K} inst={inst} lda={lda} ldb={ldb} ldc={ldc}", flush=True)
            A, B = synth.make_custom(kind, M, N, K, seed=int(rng.integers(1 << 30)), p0=float(rng.choice([0.0, 0.3, 0.9])))
            bufA = np.full((M, lda), 1, dtype=np.int8)
            bufA[:, :K] = A
            bufB = np.full((K, ldb), -1, dtype=np.int8)
            bufB[:, :N] = B
            Ap = lb.pack_t4(torch.from_numpy(bufA).cuda(), M, K, lda, 1)
            Bp = lb.pack_t4(torch.from_numpy(bufB).cuda(), N, K, 1, ldb)
            C = torch.full((M, ldc), 99, dtype=torch.int32, device="cuda")
            lb.lb_set_variant(5, inst)
            lb.gemm_t4_mfma(M, N, K, Ap, Bp, C, ldc)
            lb.lb_set_variant(5, -1)
            got = C.cpu().numpy()
            assert np.array_equal(got[:, :N], oracle.gemm(A, B)), n
            assert (got[:, N:] == 99).all(), n
    finally:
        lb.lb_set_variant(5, -1)


def test_t4_captured_in_a_graph_replays_exactly():
    """pack_t4 + gemm_t4_mfma on a shape whose product is two launches (289 tiles of 256 x 256: the last columns go to a
    second launch), captured once and replayed with new inputs and eager work in between."""
    M, N, K = 4100, 4300, 300
    dA = torch.zeros((M, K), dtype=torch.int8, device="cuda")
    dB = torch.zeros((K, N), dtype=torch.int8, device="cuda")
    Ap = torch.empty(lb.packed_t4_bytes(M, K), dtype=torch.uint8, device="cuda")
    Bp = torch.empty(lb.packed_t4_bytes(N, K), dtype=torch.uint8, device="cuda")
    C = torch.empty((M, N), dtype=torch.int32, device="cuda")

    def pipeline():
        lb.pack_t4(dA, M, K, K, 1, Ap)
        lb.pack_t4(dB, N, K, 1, N, Bp)
        lb.gemm_t4_mfma(M, N, K, Ap, Bp, C, N)

    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        pipeline()
    torch.cuda.current_stream().wait_stream(st)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        pipeline()
    for rep in range(3):
        A, B = synth.make_custom("tnn", M, N, K, seed=700 + rep)
        dA.copy_(torch.from_numpy(A))
        dB.copy_(torch.from_numpy(B))
        C.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B)), rep
