"""GPU parity for the fused threshold epilogue (gemm_requant): packed output bit for bit against oracle + packer."""
import sys

import numpy as np
import pytest
import torch

from oracle import bitref, oracle, requant
from paper_2205_09120_amd import binding as lb
from paper_2205_09120_amd import synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def words(t):
    return t.cpu().numpy().view(np.uint64)


SHAPES = [(1, 1, 1), (64, 64, 64), (65, 33, 130), (130, 257, 577), (512, 784, 2304), (1024, 300, 640), (7, 500, 64),
          (200, 5, 1000)]


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
@pytest.mark.parametrize("planes", [1, 2])
def test_requant_matches_oracle(kind, planes):
    rng = np.random.default_rng(17)
    for (M, N, K) in SHAPES:
        say(f"gemm_requant {kind} planes={planes} M={M} N={N} K={K}")
        A, B = synth.make_custom(kind, M, N, K, seed=M + 2 * N + 3 * K)
        C = oracle.gemm(A, B)
        s = max(1, int(C.std()))
        lo = rng.integers(-s, 1, size=M).astype(np.int32)
        hi = rng.integers(0, s + 1, size=M).astype(np.int32)
        Y = requant.requantize(C, lo, hi, planes == 2)                      # (N, M) int8
        want = (bitref.pack_ternary(Y) if planes == 2 else bitref.pack_binary(Y)).reshape(-1)
        Ap = lb.pack_a(kind, torch.from_numpy(A).cuda())
        Bp = lb.pack_b(kind, torch.from_numpy(B).cuda())
        Out = lb.gemm_requant(kind, planes, M, N, K, Ap, Bp, torch.from_numpy(lo).cuda(),
                              torch.from_numpy(hi).cuda() if planes == 2 else None)
        torch.cuda.synchronize()
        assert np.array_equal(words(Out), want), (M, N, K)


def test_requant_all_variants_and_chaining():
    """Every tile variant, and the output used directly as the right operand of a second product."""
    M, N, K = 192, 300, 448
    A, B = synth.make_custom("tnn", M, N, K, seed=9)
    C = oracle.gemm(A, B)
    lo = np.full(M, -8, dtype=np.int32)
    hi = np.full(M, 8, dtype=np.int32)
    Y = requant.requantize(C, lo, hi, True)                                 # (N, M): next layer's activations
    want = bitref.pack_ternary(Y).reshape(-1)
    Ap = lb.pack_a("tnn", torch.from_numpy(A).cuda())
    Bp = lb.pack_b("tnn", torch.from_numpy(B).cuda())
    dlo, dhi = torch.from_numpy(lo).cuda(), torch.from_numpy(hi).cuda()
    try:
        for v in list(range(lb.lb_num_variants("tnn"))) + [-1]:
            say(f"gemm_requant tnn variant {v}")
            lb.lb_set_variant("tnn", v)
            Out = lb.gemm_requant("tnn", 2, M, N, K, Ap, Bp, dlo, dhi)
            torch.cuda.synchronize()
            assert np.array_equal(words(Out), want), v
    finally:
        lb.lb_set_variant("tnn", -1)
    # second layer: W2 (F2 x M) times the re-quantized map (M x N): Out is exactly the packed B operand it needs
    W2, _ = synth.make_custom("tnn", 50, 1, M, seed=10)
    C2 = lb.gemm_tnn(50, N, M, lb.pack_a("tnn", torch.from_numpy(W2).cuda()), Out)
    torch.cuda.synchronize()
    assert np.array_equal(C2.cpu().numpy(), oracle.gemm(W2, np.ascontiguousarray(Y.T)))
