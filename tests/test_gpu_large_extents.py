"""GPU parity at extents that overflow 32-bit element or byte counts (64-bit addressing inside the kernels).

The outputs are too many to recompute on the CPU, so sampled entries are checked one by one against the oracle and
the rest through properties that hold for every entry (eq. (6): parity and range of a binary product).
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
    lb.lib()


def sample_indices(M, N, count, seed):
    rng = np.random.default_rng(seed)
    ii = rng.integers(0, M, size=count, dtype=np.int64)
    jj = rng.integers(0, N, size=count, dtype=np.int64)
    # corners, the last element, and the entries on both sides of the 2^31-th output
    edge = [(0, 0), (0, N - 1), (M - 1, 0), (M - 1, N - 1)]
    for flat in (2 ** 31 - 1, 2 ** 31, 2 ** 31 + 1):
        if flat < M * N:
            edge.append((flat // N, flat % N))
    ii[:len(edge)] = [e[0] for e in edge]
    jj[:len(edge)] = [e[1] for e in edge]
    return ii, jj


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_gemm_more_than_2_pow_31_outputs(kind):
    M, N, K = 46500, 46400, 100
    assert M * N > 2 ** 31
    say(f"gemm_{kind} M={M} N={N} K={K}: {M * N} outputs, sampled against the oracle")
    A, B = synth.make_custom(kind, M, N, K, seed=31)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    Ap, Bp = lb.pack_a(kind, dA), lb.pack_b(kind, dB)
    C = torch.full((M, N), -777, dtype=torch.int32, device="cuda")
    lb.gemm(kind, M, N, K, Ap, Bp, C, N)
    torch.cuda.synchronize()
    ii, jj = sample_indices(M, N, 50000, seed=32)
    got = C[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy()
    assert np.array_equal(got, oracle.gemm_samples(A, B, ii, jj))
    # every entry: |c| <= K; for binary operands also c = K mod 2 (eq. (6)); nothing left at the fill value
    assert int(C.abs().max()) <= K
    if kind == "bnn":
        assert bool(((C & 1) == (K & 1)).all())
    # whole rows and columns at the far end against the full oracle
    tail = C[M - 3:, :].cpu().numpy()
    assert np.array_equal(tail, oracle.gemm(np.ascontiguousarray(A[M - 3:]), B))
    right = C[:, N - 2:].cpu().numpy()
    assert np.array_equal(right, oracle.gemm(A, np.ascontiguousarray(B[:, N - 2:])))
    del C


@pytest.mark.parametrize("ternary", [True, False])
def test_pack_source_larger_than_2_pow_31_bytes(ternary):
    rows, K = 2_200_000, 1000
    assert rows * K > 2 ** 31
    say(f"pack ternary={ternary} rows={rows} K={K}: {rows * K} source bytes, depth-contiguous and depth-strided")
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    f = lb.pack_ternary if ternary else lb.pack_binary
    ref = bitref.pack_ternary if ternary else bitref.pack_binary
    planes = 2 if ternary else 1
    KW = (K + 63) // 64
    pick = np.array([0, 1, 63, 64, 65, rows // 2, 2 ** 31 // K, 2 ** 31 // K + 1, rows - 2, rows - 1], dtype=np.int64)
    tpick = torch.from_numpy(pick).cuda()

    def values(shape):
        x = torch.randint(-1, 2, shape, dtype=torch.int8, device="cuda", generator=g)
        return x if ternary else torch.where(x == 0, torch.ones_like(x), x)

    # depth-contiguous: rows x K
    X = values((rows, K))
    P = f(X, rows, K, K, 1)
    torch.cuda.synchronize()
    got = P.view(rows, KW * planes)[tpick].cpu().numpy().view(np.uint64)
    want = ref(X[tpick].cpu().numpy()).reshape(len(pick), -1)
    assert np.array_equal(got, want)
    del X, P
    # depth-strided: K x rows, string r is column r
    Y = values((K, rows))
    P = f(Y, rows, K, 1, rows)
    torch.cuda.synchronize()
    got = P.view(rows, KW * planes)[tpick].cpu().numpy().view(np.uint64)
    want = ref(np.ascontiguousarray(Y[:, tpick].cpu().numpy().T)).reshape(len(pick), -1)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
@pytest.mark.parametrize("M,N,K", [(3, 5, 2 ** 22 + 3), (70, 4, 2 ** 20 + 1), (2, 200, 2 ** 19 + 65)])
def test_gemm_very_deep(kind, M, N, K):
    """Depths of millions of positions: tens of thousands of depth words per string, tiled and depth-split kernels."""
    say(f"gemm_{kind} deep M={M} N={N} K={K}")
    A, B = synth.make_custom(kind, M, N, K, seed=K % 1000)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    C = lb.gemm(kind, M, N, K, lb.pack_a(kind, dA), lb.pack_b(kind, dB))
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B))


@pytest.mark.parametrize("K", [131071, 131056])
def test_i8_mfma_at_the_depth_limit(K):
    """The largest depth int32 accumulation of int8 products allows (eq. (4) with p = 8 and a 32-bit accumulator):
    full-range values, all products of one sign in the first row / column."""
    M, N = 65, 36
    say(f"gemm_i8_mfma at the depth limit M={M} N={N} K={K}")
    rng = np.random.default_rng(K)
    A = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
    B = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    A[0, :] = -128
    B[:, 0] = -128                      # C[0][0] = K * 2^14, the largest value the accumulator must hold
    C = lb.gemm_i8_mfma(M, N, K, torch.from_numpy(A).cuda(), K, torch.from_numpy(B).cuda(), N)
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    assert got[0, 0] == K * 16384
    assert np.array_equal(got, oracle.gemm(A, B))
    with pytest.raises(lb.LowbitError) as e:
        lb.gemm_i8_mfma(M, N, 131072, torch.from_numpy(A).cuda(), 131072, torch.from_numpy(B).cuda(), N)
    assert e.value.status == lb.LB_EOVERFLOW


def test_im2col_packed_more_than_2_pow_31_pieces():
    """A binary lowering whose output has more than 2^31 eight-byte pieces (64-bit index arithmetic in the kernel):
    10 maps of 1000 x 1000 x 64, a 15 x 15 window -> 10 M strings of depth 14400 (18 GB).  Sampled output strings,
    among them the corners, the last one and the ones around piece 2^31, are rebuilt by the im2col oracle from the
    window of the unpacked map."""
    from oracle import im2col as im2col_ref
    nb, H, W, C, k, pad = 10, 1000, 1000, 64, 15, 7
    taps = k * k
    assert nb * H * W * taps > 2 ** 31
    say(f"im2col_packed binary {nb}x{H}x{W}x{C} window {k}x{k}: {nb * H * W * taps} pieces")
    rng = np.random.default_rng(99)
    fmap = rng.integers(0, 2, size=(nb, H, W, C), dtype=np.int8)
    fmap = (fmap * 2 - 1).astype(np.int8)
    d = torch.from_numpy(fmap).cuda()
    Fp = lb.pack_binary(d, nb * H * W, C, C, 1)
    del d
    Bp = lb.im2col_packed(Fp, 1, nb, H, W, C, k, k, 1, 1, pad, pad)
    torch.cuda.synchronize()
    assert Bp.numel() == nb * H * W * taps
    n_mid = 2 ** 31 // taps
    pick = np.concatenate([np.array([0, W - 1, (H - 1) * W, H * W - 1, nb * H * W - 1, n_mid - 1, n_mid, n_mid + 1]),
                           rng.integers(0, nb * H * W, size=600)])
    got = Bp.view(nb * H * W, taps)[torch.from_numpy(pick).cuda()].cpu().numpy().view(np.uint64)
    for row, n in zip(got, pick):
        b, r = divmod(int(n), H * W)
        oy, ox = divmod(r, W)
        win = np.zeros((1, k, k, C), dtype=np.int8)                       # the window, zero outside the map
        y0, y1, x0, x1 = max(oy - pad, 0), min(oy + pad + 1, H), max(ox - pad, 0), min(ox + pad + 1, W)
        win[0, y0 - (oy - pad):y1 - (oy - pad), x0 - (ox - pad):x1 - (ox - pad), :] = fmap[b, y0:y1, x0:x1, :]
        col = im2col_ref.im2col(win, k, k)                                # (k*k*C, 1): the string of this pixel
        # padding positions hold 0 in the unpacked column; the packed binary string has bit 0 there as well
        want = bitref.pack_binary(np.ascontiguousarray(col.T)).reshape(-1)
        assert np.array_equal(row, want), int(n)
    del Bp


def test_matrix_core_products_more_than_2_pow_31_outputs():
    """gemm_t4_mfma and gemm_u4_mfma on 46500 x 46400 outputs: sampled entries against the oracle, every entry of the
    4-bit float product against gemm_bnn's output (itself checked above), and the range every entry must lie in."""
    M, N, K = 46500, 46400, 100
    say(f"gemm_t4_mfma / gemm_u4_mfma M={M} N={N} K={K}: {M * N} outputs")
    A, B = synth.make_custom("bnn", M, N, K, seed=31)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    ii, jj = sample_indices(M, N, 50000, seed=33)
    di, dj = torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()
    want = oracle.gemm_samples(A, B, ii, jj)
    C = torch.full((M, N), -777, dtype=torch.int32, device="cuda")
    lb.gemm_t4_mfma(M, N, K, lb.pack_t4(dA, M, K, K, 1), lb.pack_t4(dB, N, K, 1, N), C, N)
    torch.cuda.synchronize()
    assert np.array_equal(C[di, dj].cpu().numpy(), want)
    assert int(C.abs().max()) <= K and int((C & 1).sum()) == 0          # K even: every binary product is even
    C2 = torch.empty_like(C)
    lb.gemm("bnn", M, N, K, lb.pack_a("bnn", dA), lb.pack_b("bnn", dB), C2, N)
    torch.cuda.synchronize()
    assert torch.equal(C, C2)
    del C2
    # 4-bit unsigned: values {0, 2} with zero point 1 are the same +-1 matrices
    uA, uB = (dA + 1).to(torch.uint8), (dB + 1).to(torch.uint8)
    Ap, sA = lb.pack_u4(uA, M, K, K, 1)
    Bp, sB = lb.pack_u4(uB, N, K, 1, N)
    C.fill_(-777)
    lb.gemm_u4_mfma(M, N, K, Ap, sA, Bp, sB, 1, 1, C, N)
    torch.cuda.synchronize()
    assert np.array_equal(C[di, dj].cpu().numpy(), want)
    assert int(C.abs().max()) <= K and int((C & 1).sum()) == 0
