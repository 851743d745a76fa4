"""Every entry point only enqueues kernels on the caller's stream, so a sequence of calls can be captured into a
HIP graph.  The graph is replayed several times with new input values between the replays, with the program's own
eager work and synchronisations in between, and every replay is checked against the CPU oracle."""
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


def test_captured_pipeline_replays_exactly():
    assert torch.cuda.is_available()
    M, N, K = 96, 200, 330
    say(f"graph capture: pack + gemm_tnn + gemm_requant + gemm_i8_mfma + grouped launch, M={M} N={N} K={K}")
    A0, B0 = synth.make_custom("tnn", M, N, K, seed=1)
    dA, dB = torch.from_numpy(A0).cuda(), torch.from_numpy(B0).cuda()
    Ap = torch.empty(lb.packed_ternary_bytes(M, K) // 8, dtype=torch.int64, device="cuda")
    Bp = torch.empty(lb.packed_ternary_bytes(N, K) // 8, dtype=torch.int64, device="cuda")
    C = torch.empty((M, N), dtype=torch.int32, device="cuda")
    C8 = torch.empty((M, N), dtype=torch.int32, device="cuda")
    lo = torch.full((M,), -5, dtype=torch.int32, device="cuda")
    hi = torch.full((M,), 5, dtype=torch.int32, device="cuda")
    Q = torch.empty(lb.packed_ternary_bytes(N, M) // 8, dtype=torch.int64, device="cuda")
    # a small group that reuses the packed operands twice (two problems writing to two outputs)
    Cg = [torch.empty((M, N), dtype=torch.int32, device="cuda") for _ in range(2)]
    grp = lb.GemmGroup("tnn", [(Ap, Bp), (Ap, Bp)], [(M, N, K), (M, N, K)], Cg)

    def pipeline():
        lb.pack_ternary(dA, M, K, K, 1, Ap)
        lb.pack_ternary(dB, N, K, 1, N, Bp)
        lb.gemm_tnn(M, N, K, Ap, Bp, C, N)
        lb.gemm_requant("tnn", 2, M, N, K, Ap, Bp, lo, hi, Q)
        lb.gemm_i8_mfma(M, N, K, dA, K, dB, N, C8, N)
        grp.run()

    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        pipeline()                                    # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(st)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        pipeline()
    for rep in range(4):
        A, B = synth.make_custom("tnn", M, N, K, seed=100 + rep)
        dA.copy_(torch.from_numpy(A))                 # eager work between the replays
        dB.copy_(torch.from_numpy(B))
        for t in (C, C8, Q, *Cg):
            t.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want = oracle.gemm(A, B)
        assert np.array_equal(C.cpu().numpy(), want), rep
        assert np.array_equal(C8.cpu().numpy(), want), rep
        for c in Cg:
            assert np.array_equal(c.cpu().numpy(), want), rep
        Y = requant.requantize(want, lo.cpu().numpy(), hi.cpu().numpy(), True)
        assert np.array_equal(Q.cpu().numpy().view(np.uint64), bitref.pack_ternary(Y).reshape(-1)), rep
        assert np.array_equal(Ap.cpu().numpy().view(np.uint64), bitref.pack_ternary(A).reshape(-1)), rep
