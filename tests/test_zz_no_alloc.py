"""gemm_grouped_static (the grouped launch whose table lives in an array inside the library, for callers that cannot
allocate) against gemm_grouped on the same planned table, and both against the CPU oracle: bit-exact, two calls in a
row, the second on a smaller group, so that whatever the first call left in the array cannot leak into the second."""
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


def _group(kind, shapes, seed0):
    mats, packed = [], []
    for idx, (M, N, K) in enumerate(shapes):
        A, B = synth.make_custom(kind, M, N, K, seed=seed0 + idx)
        mats.append((A, B))
        packed.append((lb.pack_a(kind, torch.from_numpy(A).cuda()), lb.pack_b(kind, torch.from_numpy(B).cuda())))
    return mats, packed


def _fresh(shapes, fill):
    return [torch.full((M, N), fill, dtype=torch.int32, device="cuda") for (M, N, K) in shapes]


@pytest.mark.parametrize("kind", ["tnn", "tbn", "bnn"])
def test_grouped_static_matches_grouped_twice_second_smaller(kind):
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lb.lib()
    grid = list(synth.paper_shape_grid())                      # 64 products: several upload pieces
    small = [(33, 47, 1000), (200, 3, 129), (17, 65, 65)]      # fits one piece, both orientations, ragged
    for shapes, seed0 in ((grid, 6000), (small, 6100)):
        say(f"gemm_grouped_static {kind}: {len(shapes)} problems, first {shapes[0]}")
        mats, packed = _group(kind, shapes, seed0)
        want = lb.GemmGroup(kind, packed, shapes, _fresh(shapes, -777))
        want.run()
        got = lb.GemmGroup(kind, packed, shapes, _fresh(shapes, -555))
        assert got.table_host.numel() <= lb.gemm_grouped_static_max_bytes()
        got.run_static()
        torch.cuda.synchronize()
        for (A, B), Cw, Cg, shp in zip(mats, want.Cs, got.Cs, shapes):
            assert torch.equal(Cw, Cg), (kind, shp)
            assert np.array_equal(Cg.cpu().numpy(), oracle.gemm(A, B)), (kind, shp)


def test_grouped_static_host_table_may_be_reused_after_the_call():
    """The table travels inside kernel arguments: overwriting the host copy right after the call changes nothing."""
    lb.lib()
    shapes = [(72, 24, 128), (120, 96, 512), (5, 300, 64)]
    mats, packed = _group("tnn", shapes, 6200)
    g = lb.GemmGroup("tnn", packed, shapes, _fresh(shapes, -1))
    keep = g.table_host.clone()
    lb.gemm_grouped_static("tnn", len(shapes), g.table_host, g.workgroups)
    g.table_host.zero_()
    torch.cuda.synchronize()
    for (A, B), C in zip(mats, g.Cs):
        assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B))
    # a table beyond the array is refused before anything is enqueued
    with pytest.raises(lb.LowbitError) as e:
        lb.gemm_grouped_static("tnn", len(shapes), keep[:16].contiguous(), g.workgroups)
    assert e.value.status == lb.LB_EINVAL
