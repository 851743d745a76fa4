"""Pins for the 4-bit operand reference packer (no GPU): the 6-bit code table against the published properties of the
element type, hand-computed byte positions, the round trip, and the zero-point identity of eq. (3) with the packer's sums."""
import numpy as np
import pytest

from oracle import oracle, u4ref


def test_code_values_match_the_published_element_type():
    """1 sign / 2 exponent / 3 mantissa bits, bias 1: largest value 7.5, smallest normal 1.0, subnormals in steps of
    0.125 up to 0.875, two zeros."""
    vals = [u4ref.e2m3_value(c) for c in range(64)]
    assert max(vals) == 7.5 and min(vals) == -7.5
    assert vals[0] == 0.0 and vals[32] == 0.0
    assert [vals[c] for c in range(1, 8)] == [0.125 * m for m in range(1, 8)]
    assert vals[8] == 1.0 and vals[31] == 7.5 and vals[0b010000] == 2.0 and vals[0b011000] == 4.0
    assert sorted(set(abs(v) for v in vals)) == sorted(set(
        [m / 8 for m in range(8)] + [(1 + m / 8) * s for s in (1, 2, 4) for m in range(8)]))


def test_code_table_by_hand():
    # v/2 = 0, .5 (subnormal 4/8), 1, 1.5, 2, 2.5, 3, 3.5, 4, 4.5, ... 7.5
    assert u4ref.CODES.tolist() == [0, 4, 8, 12, 16, 18, 20, 22, 24, 25, 26, 27, 28, 29, 30, 31]


def test_sizes():
    assert u4ref.packed_u4_bytes(1, 1) == 2 * 1536
    assert u4ref.packed_u4_bytes(32, 128) == 2 * 1536
    assert u4ref.packed_u4_bytes(33, 129) == 2 * 4 * 1536
    assert u4ref.packed_u4_bytes(1024, 4608) == 32 * 72 * 1536


def test_single_element_positions_by_hand():
    P, s = u4ref.pack_u4(np.array([[15]], dtype=np.uint8))
    assert P.size == 3072 and P[0] == 31 and P[1:].sum() == 0 and s.tolist() == [15]

    X = np.zeros((34, 98), dtype=np.uint8)
    X[33, 97] = 9                      # row block 1, slot row 1; depth block 1, half 1, position 1 -> bits 6..11
    P, s = u4ref.pack_u4(X)
    assert P.size == 2 * 2 * 1536
    off = (1 * 2 + 1) * 1536 + 0 * 512 + (32 + 1) * 8
    assert P[off] == 0x40 and P[off + 1] == 0x06            # 25 << 6 = 0x640
    assert int(P.astype(np.int64).sum()) == 0x40 + 0x06
    assert s[33] == 9 and s.sum() == 9

    X = np.zeros((1, 64), dtype=np.uint8)
    X[0, 42] = 15                      # half 1, position 10 -> bits 60..65: straddles planes 0 and 1
    P, _ = u4ref.pack_u4(X)
    slot = 32
    assert P[0 * 512 + slot * 8 + 7] == 0xF0 and P[1 * 512 + slot * 8] == 0x01
    assert int(P.astype(np.int64).sum()) == 0xF0 + 0x01


@pytest.mark.parametrize("rows,K", [(1, 1), (5, 63), (32, 128), (33, 129), (70, 300)])
def test_round_trip(rows, K):
    rng = np.random.default_rng(rows * 1000 + K)
    X = rng.integers(0, 16, size=(rows, K), dtype=np.uint8)
    P, s = u4ref.pack_u4(X)
    assert P.size == u4ref.packed_u4_bytes(rows, K)
    assert np.array_equal(u4ref.unpack_u4(P, rows, K), X)
    assert np.array_equal(s, X.sum(axis=1, dtype=np.int64).astype(np.int32))


def test_zero_point_identity_with_packer_sums():
    """eq. (3): sum (a - zA)(b - zB) = sum a b - zB * rowsum(A) - zA * colsum(B) + K zA zB."""
    rng = np.random.default_rng(7)
    M, N, K = 9, 11, 77
    A = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
    B = rng.integers(0, 16, size=(K, N), dtype=np.uint8)
    _, sa = u4ref.pack_u4(A)
    _, sb = u4ref.pack_u4(np.ascontiguousarray(B.T))
    for zA, zB in [(0, 0), (8, 8), (3, 15)]:
        want = oracle.gemm_u8_zero_point(A, B, zA, zB)
        raw = A.astype(np.int64) @ B.astype(np.int64)
        got = raw - zB * sa.astype(np.int64)[:, None] - zA * sb.astype(np.int64)[None, :] + K * zA * zB
        assert np.array_equal(want, got.astype(np.int32))
