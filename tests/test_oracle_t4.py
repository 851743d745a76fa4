"""Pins for the 4-bit float operand reference packer (no GPU): the code values against the published properties of the
element type, hand-computed byte positions, the round trip through an independent decoder."""
import numpy as np
import pytest

from oracle import t4ref


def test_code_values_match_the_published_element_type():
    """1 sign / 2 exponent / 1 mantissa bit, bias 1: magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6."""
    vals = [t4ref.e2m1_value(c) for c in range(16)]
    assert vals[:8] == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert vals[8:] == [-v for v in vals[:8]]
    assert max(vals) == 6.0


def test_codes_by_hand():
    assert t4ref.code_of(0) == 0b0000 and t4ref.code_of(1) == 0b0010 and t4ref.code_of(-1) == 0b1010


def test_sizes():
    assert t4ref.packed_t4_bytes(1, 1) == 2 * 1024
    assert t4ref.packed_t4_bytes(33, 129) == 2 * 4 * 1024
    assert t4ref.packed_t4_bytes(1024, 4608) == 32 * 72 * 1024


def test_single_element_positions_by_hand():
    P = t4ref.pack_t4(np.array([[-1]], dtype=np.int8))
    assert P.size == 2048 and P[0] == 0x0A and P[1:].sum() == 0

    X = np.zeros((34, 98), dtype=np.int8)
    X[33, 97] = 1                      # row block 1, slot row 1; depth block 1, half 1, position 1 -> bits 4..7
    P = t4ref.pack_t4(X)
    assert P.size == 2 * 2 * 1024
    off = (1 * 2 + 1) * 1024 + (32 + 1) * 16
    assert P[off] == 0x20 and int(P.astype(np.int64).sum()) == 0x20

    X = np.zeros((1, 64), dtype=np.int8)
    X[0, 47] = -1                      # half 1, position 15 -> bits 60..63: high nibble of byte 7 of slot 32
    P = t4ref.pack_t4(X)
    assert P[32 * 16 + 7] == 0xA0 and int(P.astype(np.int64).sum()) == 0xA0


def test_values_are_taken_by_sign():
    X = np.array([[5, -7, 0, 1, -1, 127, -128]], dtype=np.int8)
    assert np.array_equal(t4ref.unpack_t4(t4ref.pack_t4(X), 1, 7), np.sign(X).astype(np.int8))


@pytest.mark.parametrize("rows,K", [(1, 1), (5, 63), (32, 128), (33, 129), (70, 300)])
def test_round_trip(rows, K):
    rng = np.random.default_rng(rows * 1000 + K)
    X = rng.integers(-1, 2, size=(rows, K)).astype(np.int8)
    P = t4ref.pack_t4(X)
    assert P.size == t4ref.packed_t4_bytes(rows, K)
    assert np.array_equal(t4ref.unpack_t4(P, rows, K), X)
