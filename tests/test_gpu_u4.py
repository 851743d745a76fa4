"""GPU parity of the 4-bit stand-in (pack_u4 + gemm_u4_mfma) against the oracle: packed bytes and row sums bit for bit
against the reference packer, products bit for bit against the zero-point definition of eq. (3)."""
import numpy as np
import pytest
import torch

from oracle import oracle, u4ref
from paper_2205_09120_amd import binding as lb

pytestmark = pytest.mark.gpu


def _draw(seed, M, N, K, lo=0, hi=16):
    rng = np.random.default_rng(seed)
    return (rng.integers(lo, hi, size=(M, K), dtype=np.uint8), rng.integers(lo, hi, size=(K, N), dtype=np.uint8))


def _pack_both(A, B):
    M, K = A.shape
    N = B.shape[1]
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    Ap, sA = lb.pack_u4(dA, M, K, K, 1)
    Bp, sB = lb.pack_u4(dB, N, K, 1, N)
    return Ap, sA, Bp, sB


@pytest.mark.parametrize("rows,K", [(1, 1), (5, 63), (32, 128), (33, 129), (70, 300), (257, 1000)])
def test_pack_u4_matches_reference_packer(rows, K):
    rng = np.random.default_rng(rows * 7 + K)
    X = rng.integers(0, 16, size=(rows, K), dtype=np.uint8)
    want, wsum = u4ref.pack_u4(X)
    got, gsum = lb.pack_u4(torch.from_numpy(X).cuda(), rows, K, K, 1)
    assert np.array_equal(got.cpu().numpy(), want)
    assert np.array_equal(gsum.cpu().numpy(), wsum)
    # the same matrix handed over depth-strided (as the K x rows right operand of a product)
    XT = np.ascontiguousarray(X.T)
    got, gsum = lb.pack_u4(torch.from_numpy(XT).cuda(), rows, K, 1, rows)
    assert np.array_equal(got.cpu().numpy(), want)
    assert np.array_equal(gsum.cpu().numpy(), wsum)


def test_pack_u4_leading_dimension_and_high_nibble_ignored():
    rng = np.random.default_rng(5)
    rows, K, ld = 45, 200, 211
    buf = rng.integers(0, 256, size=(rows, ld), dtype=np.uint8)       # high nibbles set: only the low four bits count
    want, wsum = u4ref.pack_u4(buf[:, :K] & 15)
    got, gsum = lb.pack_u4(torch.from_numpy(buf).cuda(), rows, K, ld, 1)
    assert np.array_equal(got.cpu().numpy(), want)
    assert np.array_equal(gsum.cpu().numpy(), wsum)


# the last one has a partial last round of 256 x 256 tiles (289 tiles): two launches, the second with small tiles
SHAPES = [(1, 1, 1), (3, 5, 7), (64, 64, 128), (65, 33, 129), (100, 260, 300), (256, 256, 512), (300, 520, 1000),
          (513, 130, 4608), (4100, 4300, 2100)]


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("inst", [-1, 0, 1, 2, 3])
def test_gemm_u4_matches_oracle(M, N, K, inst):
    A, B = _draw(M * 31 + N * 7 + K, M, N, K)
    Ap, sA, Bp, sB = _pack_both(A, B)
    lb.lb_set_variant(5, inst)
    try:
        for zA, zB in [(0, 0), (8, 7), (15, 1)]:
            C = lb.gemm_u4_mfma(M, N, K, Ap, sA, Bp, sB, zA, zB)
            assert np.array_equal(C.cpu().numpy(), oracle.gemm_u8_zero_point(A, B, zA, zB)), (zA, zB)
    finally:
        lb.lb_set_variant(5, -1)


def test_gemm_u4_leading_dimension_of_c():
    M, N, K, ldc = 70, 90, 256, 101
    A, B = _draw(11, M, N, K)
    Ap, sA, Bp, sB = _pack_both(A, B)
    C = torch.full((M, ldc), -7, dtype=torch.int32, device="cuda")
    lb.gemm_u4_mfma(M, N, K, Ap, sA, Bp, sB, 3, 4, C, ldc)
    got = C.cpu().numpy()
    assert np.array_equal(got[:, :N], oracle.gemm_u8_zero_point(A, B, 3, 4))
    assert (got[:, N:] == -7).all()


def test_gemm_u4_largest_sums_are_exact():
    """All values 15 at a depth close to the limit: every partial sum stays an exact fp32 integer (225 K < 2^24)."""
    M, N, K = 40, 50, 74565
    A = np.full((M, K), 15, dtype=np.uint8)
    B = np.full((K, N), 15, dtype=np.uint8)
    rng = np.random.default_rng(2)
    A[rng.integers(0, M, 200), rng.integers(0, K, 200)] = 14       # a few odd ones so the low bits are exercised
    B[rng.integers(0, K, 200), rng.integers(0, N, 200)] = 1
    Ap, sA, Bp, sB = _pack_both(A, B)
    for zA, zB in [(0, 0), (15, 15)]:
        C = lb.gemm_u4_mfma(M, N, K, Ap, sA, Bp, sB, zA, zB)
        assert np.array_equal(C.cpu().numpy(), oracle.gemm_u8_zero_point(A, B, zA, zB))


def test_gemm_u4_headline_shape_sampled():
    """cfg4's shape (1024 x 50176 x 4608) in the launch configuration the benchmark times; 4000 sampled outputs and the
    first 64 rows of a column block against the oracle."""
    M, N, K = 1024, 50176, 4608
    rng = np.random.default_rng(44)
    A = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
    B = rng.integers(0, 16, size=(K, N), dtype=np.uint8)
    Ap, sA, Bp, sB = _pack_both(A, B)
    zA, zB = 8, 8
    C = lb.gemm_u4_mfma(M, N, K, Ap, sA, Bp, sB, zA, zB).cpu().numpy()
    ii = rng.integers(0, M, 4000)
    jj = rng.integers(0, N, 4000)
    # (a - 8)(b - 8) on int8 operands is the plain product the sampled oracle computes
    As = (A.astype(np.int16) - zA).astype(np.int8)
    Bs = (B.astype(np.int16) - zB).astype(np.int8)
    assert np.array_equal(C[ii, jj], oracle.gemm_samples(As, Bs, ii, jj))
    cols = slice(50176 - 300, 50176)
    assert np.array_equal(C[:64, cols], oracle.gemm(np.ascontiguousarray(As[:64]), np.ascontiguousarray(Bs[:, cols])))


def test_u4_random_sweep():
    """Seeded random shapes, instances, zero points, leading dimensions and source layouts."""
    rng = np.random.default_rng(2024)
    try:
        for n in range(1, 161):
            r = rng.random()
            if r < 0.2:
                M, N, K = int(rng.integers(1, 40)), int(np.exp(rng.uniform(0, np.log(3000)))), int(np.exp(rng.uniform(0, np.log(20000))))
            elif r < 0.4:
                M, N, K = int(np.exp(rng.uniform(0, np.log(3000)))), int(rng.integers(1, 40)), int(np.exp(rng.uniform(0, np.log(20000))))
            else:
                M, N, K = (int(np.exp(rng.uniform(0, np.log(1200)))) for _ in range(3))
            inst = int(rng.integers(-1, lb.lb_num_variants(5)))
            zA, zB = int(rng.integers(0, 16)), int(rng.integers(0, 16))
            lda, ldb, ldc = K + int(rng.choice([0, 1, 16, 5])), N + int(rng.choice([0, 1, 4, 7])), N + int(rng.choice([0, 3]))
            a_strided = bool(rng.integers(0, 2))          # A handed over as K x M (depth-strided) instead
            print(f"[{n}] u4 M={M} N={N} K={K} inst={inst} z=({zA},{zB}) lda={lda} ldb={ldb} ldc={ldc} a_strided={a_strided}",
                  flush=True)
            A = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
            B = rng.integers(0, 16, size=(K, N), dtype=np.uint8)
            bufB = np.full((K, ldb), 9, dtype=np.uint8)
            bufB[:, :N] = B
            if a_strided:
                bufA = np.full((K, M + 3), 7, dtype=np.uint8)
                bufA[:, :M] = A.T
                Ap, sA = lb.pack_u4(torch.from_numpy(bufA).cuda(), M, K, 1, M + 3)
            else:
                bufA = np.full((M, lda), 7, dtype=np.uint8)
                bufA[:, :K] = A
                Ap, sA = lb.pack_u4(torch.from_numpy(bufA).cuda(), M, K, lda, 1)
            Bp, sB = lb.pack_u4(torch.from_numpy(bufB).cuda(), N, K, 1, ldb)
            if M * K <= 60000:
                want_p, want_s = u4ref.pack_u4(A)
                assert np.array_equal(Ap.cpu().numpy(), want_p) and np.array_equal(sA.cpu().numpy(), want_s), n
            C = torch.full((M, ldc), 99, dtype=torch.int32, device="cuda")
            lb.lb_set_variant(5, inst)
            lb.gemm_u4_mfma(M, N, K, Ap, sA, Bp, sB, zA, zB, C, ldc)
            lb.lb_set_variant(5, -1)
            got = C.cpu().numpy()
            assert np.array_equal(got[:, :N], oracle.gemm_u8_zero_point(A, B, zA, zB)), n
            assert (got[:, N:] == 99).all(), n
    finally:
        lb.lb_set_variant(5, -1)


def test_u4_captured_in_a_graph_replays_exactly():
    """pack_u4 (which clears the row sums with a fill kernel, not a memset) and gemm_u4_mfma only enqueue kernels:
    captured once, replayed with new inputs and eager work in between, every replay checked against the oracle."""
    M, N, K = 150, 300, 700
    dA = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
    dB = torch.zeros((K, N), dtype=torch.uint8, device="cuda")
    Ap = torch.empty(lb.packed_u4_bytes(M, K), dtype=torch.uint8, device="cuda")
    Bp = torch.empty(lb.packed_u4_bytes(N, K), dtype=torch.uint8, device="cuda")
    sA = torch.empty(M, dtype=torch.int32, device="cuda")
    sB = torch.empty(N, dtype=torch.int32, device="cuda")
    C = torch.empty((M, N), dtype=torch.int32, device="cuda")

    def pipeline():
        lb.pack_u4(dA, M, K, K, 1, Ap, sA)
        lb.pack_u4(dB, N, K, 1, N, Bp, sB)
        lb.gemm_u4_mfma(M, N, K, Ap, sA, Bp, sB, 5, 9, C, N)

    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        pipeline()
    torch.cuda.current_stream().wait_stream(st)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        pipeline()
    for rep in range(4):
        A, B = _draw(500 + rep, M, N, K)
        dA.copy_(torch.from_numpy(A))
        dB.copy_(torch.from_numpy(B))
        C.fill_(-1)
        sA.fill_(123)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), oracle.gemm_u8_zero_point(A, B, 5, 9)), rep
        assert np.array_equal(sA.cpu().numpy(), A.sum(axis=1, dtype=np.int64).astype(np.int32)), rep
