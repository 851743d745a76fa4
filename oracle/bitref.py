"""The paper's encodings and bitwise product formulas on the CPU.  TEST INFRASTRUCTURE ONLY.

Two things live here, both written from Section III-A of the paper:

1. The reference packer / unpacker.  It fixes, bit for bit, the packed operand
   format that the library's pack_binary / pack_ternary must produce:
     * a matrix is packed as `rows` bit strings along the depth k;
     * word w of a bit string holds depth positions 64w .. 64w+63, position k in
       bit (k mod 64) counted from the least significant bit;
     * binary  (+1 -> bit 0, -1 -> bit 1):  one uint64 per word,  dst[r*KW + w];
     * ternary (+1 -> (1,0), 0 -> (0,0), -1 -> (0,1)):  the plus word and the minus
       word of one depth word are adjacent,  dst[(r*KW + w)*2 + {0: plus, 1: minus}];
     * positions k >= K of the last word are 0 in every plane.
   Values outside the legal sets are mapped by sign (x > 0 plus, x < 0 minus; binary:
   x < 0 -> 1), so the invalid code (1,1) is never produced.

2. gemm_bitwise(): the product evaluated the way the paper states it -- eq. (6) for
   binary operands (k - 2 * popcount(a xor b)) and eq. (7) with the plus/minus
   product formulas of Section III-A for ternary and ternary-binary operands --
   one 64-bit word at a time with Python integers.  It is slow and only meant for
   small cases: it ties the packed format and the formulas to the plain definition
   computed by gemm_oracle.c.
"""
from __future__ import annotations

import numpy as np


def kwords(K: int) -> int:
    return (K + 63) // 64


def _bitplane_words(bits: np.ndarray) -> np.ndarray:
    """bits: (rows, K) of 0/1 -> (rows, KW) uint64, LSB-first within each word."""
    rows, K = bits.shape
    KW = kwords(K)
    padded = np.zeros((rows, KW * 64), dtype=np.uint8)
    padded[:, :K] = bits
    by = np.packbits(padded, axis=1, bitorder="little")  # (rows, KW*8) bytes, byte b holds positions 8b..8b+7
    return np.ascontiguousarray(by).view("<u8").reshape(rows, KW)


def pack_binary(X: np.ndarray) -> np.ndarray:
    """X: (rows, K) int8, depth along axis 1 -> (rows, KW) uint64."""
    return _bitplane_words((X < 0).astype(np.uint8))


def pack_ternary(X: np.ndarray) -> np.ndarray:
    """X: (rows, K) int8 -> (rows, KW, 2) uint64 with [...,0] = plus plane, [...,1] = minus plane."""
    plus = _bitplane_words((X > 0).astype(np.uint8))
    minus = _bitplane_words((X < 0).astype(np.uint8))
    return np.ascontiguousarray(np.stack([plus, minus], axis=-1))


def _unpack_plane(W: np.ndarray, K: int) -> np.ndarray:
    rows = W.shape[0]
    by = np.ascontiguousarray(W.astype("<u8")).view(np.uint8).reshape(rows, -1)
    return np.unpackbits(by, axis=1, bitorder="little")[:, :K]


def unpack_binary(W: np.ndarray, K: int) -> np.ndarray:
    b = _unpack_plane(W, K)
    return (1 - 2 * b.astype(np.int8)).astype(np.int8)


def unpack_ternary(W: np.ndarray, K: int) -> np.ndarray:
    p = _unpack_plane(W[..., 0], K).astype(np.int8)
    m = _unpack_plane(W[..., 1], K).astype(np.int8)
    if np.any(p & m):
        raise ValueError("invalid ternary code (1,1)")
    return (p - m).astype(np.int8)


def _popc(x: int) -> int:
    return bin(x).count("1")


_MASK = (1 << 64) - 1


def dot_bnn(aw, bw, K: int) -> int:
    """eq. (6): c = k - 2 * sum_t (a^b_t xor b^b_t), on packed words."""
    return K - 2 * sum(_popc(int(a) ^ int(b)) for a, b in zip(aw, bw))


def dot_tnn(ap, am, bp, bm) -> int:
    """eq. (7) with z+ = (x+ & y+) | (x- & y-), z- = (x+ & y-) | (x- & y+)."""
    c = 0
    for xp, xm, yp, ym in zip(ap, am, bp, bm):
        xp, xm, yp, ym = int(xp), int(xm), int(yp), int(ym)
        zp = (xp & yp) | (xm & ym)
        zm = (xp & ym) | (xm & yp)
        c += _popc(zp) - _popc(zm)
    return c


def dot_tbn(ap, am, bw) -> int:
    """eq. (7) with z+ = (x+ | y) & (x- | ~y), z- = (x+ | ~y) & (x- | y)  (y = binary code word)."""
    c = 0
    for xp, xm, y in zip(ap, am, bw):
        xp, xm, y = int(xp), int(xm), int(y)
        ny = ~y & _MASK
        zp = (xp | y) & (xm | ny)
        zm = (xp | ny) & (xm | y)
        c += _popc(zp) - _popc(zm)
    return c


def gemm_bitwise(kind: str, A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C = A B through the packed format and the paper's bit formulas.  A: M x K, B: K x N (int8)."""
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    Bt = np.ascontiguousarray(B.T)
    C = np.zeros((M, N), dtype=np.int32)
    if kind == "bnn":
        Ap, Bp = pack_binary(A), pack_binary(Bt)
        for i in range(M):
            for j in range(N):
                C[i, j] = dot_bnn(Ap[i], Bp[j], K)
    elif kind == "tnn":
        Ap, Bp = pack_ternary(A), pack_ternary(Bt)
        for i in range(M):
            for j in range(N):
                C[i, j] = dot_tnn(Ap[i, :, 0], Ap[i, :, 1], Bp[j, :, 0], Bp[j, :, 1])
    elif kind == "tbn":
        Ap, Bp = pack_ternary(A), pack_binary(Bt)
        for i in range(M):
            for j in range(N):
                C[i, j] = dot_tbn(Ap[i, :, 0], Ap[i, :, 1], Bp[j])
    else:
        raise ValueError(kind)
    return C
