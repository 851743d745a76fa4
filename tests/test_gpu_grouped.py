"""GPU parity of the grouped launch (many small products in one grid) against the CPU oracle, bit-exact.

The workload is the paper's own timing grid (Section IV-B: 4 heights x 4 widths x 4 depths) plus groups of ragged,
empty and mixed-orientation problems.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import oracle
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


def build_group(kind, shapes, seed0, ldc_extra=0):
    mats, packed, Cs = [], [], []
    for idx, (M, N, K) in enumerate(shapes):
        A, B = synth.make_custom(kind, max(M, 1), max(N, 1), K, seed=seed0 + idx)
        A, B = A[:M], B[:, :N]
        mats.append((A, B))
        dA, dB = torch.from_numpy(np.ascontiguousarray(A)).cuda(), torch.from_numpy(np.ascontiguousarray(B)).cuda()
        Ap = lb.pack_a(kind, dA) if M else torch.empty(0, dtype=torch.int64, device="cuda")
        Bp = lb.pack_b(kind, dB) if N else torch.empty(0, dtype=torch.int64, device="cuda")
        packed.append((Ap, Bp))
        Cs.append(torch.full((M, N + ldc_extra), -777, dtype=torch.int32, device="cuda"))
    return mats, packed, Cs


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_grouped_paper_shape_grid(kind):
    shapes = list(synth.paper_shape_grid())
    say(f"gemm_grouped {kind}: the 64 shapes of the paper's grid in one launch")
    mats, packed, Cs = build_group(kind, shapes, 2000)
    g = lb.GemmGroup(kind, packed, shapes, Cs)
    g.run()
    torch.cuda.synchronize()
    for (A, B), C, shp in zip(mats, Cs, shapes):
        assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B)), shp


RAGGED = [(1, 1, 1), (16, 64, 64), (17, 65, 65), (3, 200, 63), (200, 3, 129), (64, 64, 4096), (0, 9, 64), (9, 0, 64),
          (33, 47, 1000), (130, 70, 191), (15, 63, 127), (257, 2, 64), (2, 257, 640)]


@pytest.mark.parametrize("kind", ["bnn", "tnn", "tbn"])
def test_grouped_ragged_empty_and_ldc(kind):
    say(f"gemm_grouped {kind}: ragged / empty problems, ldc > N, both orientations in one grid")
    mats, packed, Cs = build_group(kind, RAGGED, 3000, ldc_extra=5)
    g = lb.GemmGroup(kind, packed, RAGGED, Cs)
    g.run()
    g.run()  # a table may be launched any number of times
    torch.cuda.synchronize()
    for (A, B), C, (M, N, K) in zip(mats, Cs, RAGGED):
        got = C.cpu().numpy()
        if M == 0 or N == 0:
            assert np.all(got == -777)
            continue
        assert np.array_equal(got[:, :N], oracle.gemm(A, B)), (M, N, K)
        assert np.all(got[:, N:] == -777), (M, N, K)


def test_grouped_matches_single_launches_on_random_groups():
    rng = np.random.default_rng(77)
    for kind in ("bnn", "tnn", "tbn"):
        shapes = [(int(rng.integers(1, 300)), int(rng.integers(1, 300)), int(rng.integers(1, 700))) for _ in range(40)]
        say(f"gemm_grouped {kind}: 40 random shapes, first {shapes[0]}")
        mats, packed, Cs = build_group(kind, shapes, 4000)
        lb.GemmGroup(kind, packed, shapes, Cs).run()
        torch.cuda.synchronize()
        for (A, B), C, shp in zip(mats, Cs, shapes):
            assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B)), (kind, shp)


def test_grouped_empty_group_and_mismatched_table():
    say("gemm_grouped: empty group; a table planned for another count is refused by the kernel")
    lb.gemm_grouped("tnn", 0, None, 0)
    shapes = [(20, 30, 100), (40, 10, 64)]
    mats, packed, Cs = build_group("tnn", shapes, 5000)
    g = lb.GemmGroup("tnn", packed, shapes, Cs)
    # same table, wrong problem count / wrong kind: the kernel checks the header and writes nothing
    lb.gemm_grouped("tnn", 3, g.table_dev, g.workgroups)
    lb.gemm_grouped("bnn", 2, g.table_dev, g.workgroups)
    lb.gemm_grouped("tnn", 2, g.table_dev, g.workgroups + 1)
    torch.cuda.synchronize()
    for C in Cs:
        assert torch.all(C == -777)
    g.run()
    torch.cuda.synchronize()
    for (A, B), C in zip(mats, Cs):
        assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B))


# ------------------------------------------------------------------ grouped launch of the 8-bit comparator

def build_i8_group(shapes, seed0, ldc_extra=0, misalign=False):
    rng = np.random.default_rng(seed0)
    mats, pairs, Cs = [], [], []
    for (M, N, K) in shapes:
        A = rng.integers(-128, 128, (M, K), dtype=np.int8)
        B = rng.integers(-128, 128, (K, N), dtype=np.int8)
        mats.append((A, B))
        if misalign and M and N:
            # operands at odd addresses with odd leading dimensions: views into larger buffers
            bufA = torch.zeros(M * (K + 3) + 1, dtype=torch.int8, device="cuda")
            dA = bufA[1:].view(M, K + 3)[:, :K]
            dA.copy_(torch.from_numpy(A))
            bufB = torch.zeros(K * (N + 1) + 3, dtype=torch.int8, device="cuda")
            dB = bufB[3:].view(K, N + 1)[:, :N]
            dB.copy_(torch.from_numpy(B))
        else:
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        pairs.append((dA, dB))
        Cs.append(torch.full((M, N + ldc_extra), -777, dtype=torch.int32, device="cuda"))
    return mats, pairs, Cs


def test_i8_grouped_paper_shape_grid():
    shapes = list(synth.paper_shape_grid())
    say("gemm_i8_grouped: the 64 shapes of the paper's grid in one launch")
    mats, pairs, Cs = build_i8_group(shapes, 7000)
    g = lb.I8Group(pairs, shapes, Cs)
    g.run()
    torch.cuda.synchronize()
    for (A, B), C, shp in zip(mats, Cs, shapes):
        assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B)), shp


I8_RAGGED = [(1, 1, 1), (64, 64, 64), (65, 67, 66), (3, 200, 63), (200, 3, 129), (64, 64, 4096), (0, 9, 64), (9, 0, 64),
             (33, 47, 1000), (130, 70, 191), (128, 128, 131071), (257, 2, 64), (2, 257, 640), (100, 16, 48), (72, 24, 128)]


@pytest.mark.parametrize("misalign", [False, True])
def test_i8_grouped_ragged_empty_ldc_and_alignment(misalign):
    say(f"gemm_i8_grouped: ragged / empty problems, every fetch mode in one grid, ldc > N, misaligned={misalign}")
    mats, pairs, Cs = build_i8_group(I8_RAGGED, 7100, ldc_extra=3, misalign=misalign)
    g = lb.I8Group(pairs, I8_RAGGED, Cs)
    g.run()
    g.run()
    torch.cuda.synchronize()
    for (A, B), C, (M, N, K) in zip(mats, Cs, I8_RAGGED):
        got = C.cpu().numpy()
        if M == 0 or N == 0:
            assert np.all(got == -777)
            continue
        assert np.array_equal(got[:, :N], oracle.gemm(A, B)), (M, N, K)
        assert np.all(got[:, N:] == -777), (M, N, K)


def test_i8_grouped_mismatched_table_is_refused():
    say("gemm_i8_grouped: a table planned for another count or grid is refused by the kernel")
    shapes = [(20, 30, 100), (40, 10, 64)]
    mats, pairs, Cs = build_i8_group(shapes, 7200)
    g = lb.I8Group(pairs, shapes, Cs)
    lb.gemm_i8_grouped(3, g.table_dev, g.workgroups)
    lb.gemm_i8_grouped(2, g.table_dev, g.workgroups + 1)
    torch.cuda.synchronize()
    for C in Cs:
        assert torch.all(C == -777)
    g.run()
    torch.cuda.synchronize()
    for (A, B), C in zip(mats, Cs):
        assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B))
