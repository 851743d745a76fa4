"""Seeded randomized parity sweep over every entry point: kind, shape (log-uniform or uniform extents, narrow and
deep ones included), tile variant / kernel instance, leading dimensions and zero points are all drawn at random; every
result is compared with the oracle bit for bit.  Complements the targeted cases of the other GPU tests."""
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


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


@pytest.fixture(autouse=True)
def _reset_forced_variants():
    yield
    for op in ("bnn", "tnn", "tbn", 3, 4):
        lb.lb_set_variant(op, -1)


@pytest.mark.parametrize("seed,count,big", [(1, 500, False), (2, 60, True)])
def test_random_sweep(seed, count, big):
    assert torch.cuda.is_available(), "these tests need the MI355X"
    rng = np.random.default_rng(seed)

    def lu(hi):
        return int(rng.integers(1, hi + 1)) if big else int(np.exp(rng.uniform(0, np.log(hi))))

    def shape():
        r = rng.random()
        if r < 0.15: return lu(3000), int(rng.integers(1, 34)), lu(20000)       # skinny N
        if r < 0.25: return int(rng.integers(1, 34)), lu(3000), lu(20000)       # skinny M
        if r < 0.35: return lu(300), lu(300), lu(40000)                          # deep
        return lu(1500), lu(1500), lu(5000)
    for n in range(1, count + 1):
        what = rng.choice(["gemm", "gemm", "c16", "requant", "i8", "u8", "group", "pack"])
        kind = ("bnn", "tnn", "tbn")[int(rng.integers(0, 3))]
        M, N, K = shape()
        if what in ("gemm", "c16"):
            if what == "c16": K = min(K, 32767)
            v = int(rng.integers(-1, lb.lb_num_variants(kind))) if rng.random() < 0.5 else -1
            ldc = N + int(rng.choice([0, 1, 4, 13]))
            say(f"[{n}] {what} {kind} M={M} N={N} K={K} variant={v} ldc={ldc}")
            A, B = synth.make_custom(kind, M, N, K, seed=int(rng.integers(1 << 30)), p0=float(rng.choice([0.0, 0.3, 0.5, 0.9])))
            want = oracle.gemm(A, B)
            Ap, Bp = lb.pack_a(kind, dev(A)), lb.pack_b(kind, dev(B))
            lb.lb_set_variant(kind, v)
            if what == "gemm":
                C = torch.full((M, ldc), 99, dtype=torch.int32, device='cuda'); lb.gemm(kind, M, N, K, Ap, Bp, C, ldc)
            else:
                C = torch.full((M, ldc), 99, dtype=torch.int16, device='cuda'); lb.gemm_c16(kind, M, N, K, Ap, Bp, C, ldc)
            torch.cuda.synchronize(); lb.lb_set_variant(kind, -1)
            got = C.cpu().numpy()
            ok = np.array_equal(got[:, :N].astype(np.int32), want) and np.all(got[:, N:] == 99)
        elif what == "requant":
            M, N, K = min(M, 1200), min(N, 1200), min(K, 3000)
            planes = int(rng.integers(1, 3))
            v = int(rng.integers(-1, lb.lb_num_variants(kind))) if rng.random() < 0.5 else -1
            say(f"[{n}] requant {kind} planes={planes} M={M} N={N} K={K} variant={v}")
            A, B = synth.make_custom(kind, M, N, K, seed=int(rng.integers(1 << 30)))
            Cc = oracle.gemm(A, B); s = max(1, int(Cc.std()))
            lo = rng.integers(-s, 1, size=M).astype(np.int32); hi = rng.integers(0, s + 1, size=M).astype(np.int32)
            Y = requant.requantize(Cc, lo, hi, planes == 2)
            want = (bitref.pack_ternary(Y) if planes == 2 else bitref.pack_binary(Y)).reshape(-1)
            lb.lb_set_variant(kind, v)
            Out = lb.gemm_requant(kind, planes, M, N, K, lb.pack_a(kind, dev(A)), lb.pack_b(kind, dev(B)), dev(lo), dev(hi) if planes == 2 else None)
            torch.cuda.synchronize(); lb.lb_set_variant(kind, -1)
            ok = np.array_equal(Out.cpu().numpy().view(np.uint64), want)
        elif what in ("i8", "u8"):
            K = min(K, 6000)
            if rng.random() < 0.5: N = max(16, N // 16 * 16)
            if rng.random() < 0.6: K = max(64, K // 64 * 64)
            lda = K + int(rng.choice([0, 16, 3])); ldb = N + int(rng.choice([0, 16, 4, 1])); ldc = N + int(rng.choice([0, 5]))
            v = int(rng.integers(-1, lb.lb_num_variants(4))) if (what == "i8" and rng.random() < 0.5) else -1
            zA, zB = int(rng.integers(0, 256)), int(rng.integers(0, 256))
            say(f"[{n}] {what} M={M} N={N} K={K} lda={lda} ldb={ldb} ldc={ldc} variant={v} z=({zA},{zB})")
            A = np.full((M, lda), 77, dtype=np.int8); B = np.full((K, ldb), -55, dtype=np.int8)
            A[:, :K] = rng.integers(-128, 128, size=(M, K), dtype=np.int8); B[:, :N] = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
            C = torch.full((M, ldc), 99, dtype=torch.int32, device='cuda')
            if what == "i8":
                lb.lb_set_variant(4, v); lb.gemm_i8_mfma(M, N, K, dev(A), lda, dev(B), ldb, C, ldc); torch.cuda.synchronize(); lb.lb_set_variant(4, -1)
                want = oracle.gemm(np.ascontiguousarray(A[:, :K]), np.ascontiguousarray(B[:, :N]))
            else:
                lb.gemm_u8_mfma(M, N, K, dev(A.view(np.uint8)), lda, dev(B.view(np.uint8)), ldb, zA, zB, C, ldc); torch.cuda.synchronize()
                want = oracle.gemm_u8_zero_point(np.ascontiguousarray(A.view(np.uint8)[:, :K]), np.ascontiguousarray(B.view(np.uint8)[:, :N]), zA, zB)
            got = C.cpu().numpy()
            ok = np.array_equal(got[:, :N], want) and np.all(got[:, N:] == 99)
        elif what == "group":
            cnt = int(rng.integers(1, 12))
            shapes = [(int(rng.integers(0, 400)), int(rng.integers(0, 400)), lu(3000)) for _ in range(cnt)]
            say(f"[{n}] group {kind} {shapes}")
            mats, packed, Cs = [], [], []
            for (m, nn, k) in shapes:
                A, B = synth.make_custom(kind, max(m, 1), max(nn, 1), k, seed=int(rng.integers(1 << 30)))
                A, B = A[:m], B[:, :nn]; mats.append((A, B))
                packed.append((lb.pack_a(kind, dev(A)) if m else torch.empty(0, dtype=torch.int64, device='cuda'),
                               lb.pack_b(kind, dev(B)) if nn else torch.empty(0, dtype=torch.int64, device='cuda')))
                Cs.append(torch.full((m, nn + 2), -7, dtype=torch.int32, device='cuda'))
            g = lb.GemmGroup(kind, packed, shapes, Cs); g.run(); torch.cuda.synchronize()
            ok = all(np.array_equal(C.cpu().numpy()[:, :s[1]], oracle.gemm(np.ascontiguousarray(A), np.ascontiguousarray(B))) and np.all(C.cpu().numpy()[:, s[1]:] == -7)
                     for (A, B), C, s in zip(mats, Cs, shapes) if s[0] and s[1])
        else:
            rows, Kp = lu(3000), lu(20000)
            tern = bool(rng.integers(0, 2)); strided = bool(rng.integers(0, 2))
            pad = int(rng.choice([0, 1, 4, 16, 7]))
            say(f"[{n}] pack rows={rows} K={Kp} ternary={tern} strided={strided} pad={pad}")
            X = rng.integers(-1, 2, size=(rows, Kp), dtype=np.int8)
            want = (bitref.pack_ternary(X) if tern else bitref.pack_binary(X)).reshape(-1)
            f = lb.pack_ternary if tern else lb.pack_binary
            if strided:
                buf = np.zeros((Kp, rows + pad), dtype=np.int8); buf[:, :rows] = X.T
                got = f(dev(buf), rows, Kp, 1, rows + pad)
            else:
                buf = np.zeros((rows, Kp + pad), dtype=np.int8); buf[:, :Kp] = X
                got = f(dev(buf), rows, Kp, Kp + pad, 1)
            torch.cuda.synchronize()
            ok = np.array_equal(got.cpu().numpy().view(np.uint64), want)
        assert ok, f"mismatch in case {n}"
