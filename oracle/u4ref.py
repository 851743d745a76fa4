"""Reference packer for 4-bit unsigned operands of the matrix-core stand-in for the paper's U4 algorithm
(Table II, Section IV; quantized product with zero points: eq. (2) and (3)).  TEST INFRASTRUCTURE ONLY.

The product itself needs no new oracle: it is oracle.gemm_u8_zero_point on matrices whose entries lie in 0..15.
This module fixes, bit for bit, the operand format the library's pack_u4 must produce:

  * every value v in 0..15 is stored as the 6-bit floating-point code (1 sign, 2 exponent, 3 mantissa bits,
    exponent bias 1, subnormals at exponent 0 -- the "E2M3" element type of the Open Compute microscaling
    formats) whose value is v / 2; all sixteen halves 0, 0.5, ..., 7.5 are representable;
  * a matrix is packed as `rows` strings along the depth k; rows are padded to a multiple of 32 and the depth to a
    multiple of 128 with the code of 0;
  * a "fragment" is 32 rows x 64 depth positions: 64 slots of 192 bits, slot 32*h + i holding depth positions
    64*kb + 32*h + j (j = 0..31) of row 32*rb + i, position j in bits 6j .. 6j+5 of the 192-bit little-endian
    string; the fragment is stored as three planes of 64 x 8 bytes: plane p holds bits 64p .. 64p+63 of every slot
    (byte offset p*512 + slot*8);
  * fragments are ordered by row block, then depth block: byte offset (rb * KB + kb) * 1536 with KB = 2*ceil(K/128);
  * next to the packed strings goes one int32 per row: the sum of its K values (the row / column sums of eq. (3)).
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

FRAGMENT_BYTES = 1536


def e2m3_value(code: int) -> float:
    """Value of a 6-bit code: sign s, exponent e (2 bits, bias 1), mantissa m (3 bits)."""
    s, e, m = (code >> 5) & 1, (code >> 3) & 3, code & 7
    mag = (m / 8.0) if e == 0 else (2.0 ** (e - 1)) * (1.0 + m / 8.0)
    return -mag if s else mag


def code_of(v: int) -> int:
    """The code whose value is v / 2, found by search over all 64 codes (the smallest one: +0 rather than -0)."""
    for code in range(64):
        if e2m3_value(code) == v / 2.0:
            return code
    raise ValueError(f"{v}/2 has no 6-bit code")


CODES = np.array([code_of(v) for v in range(16)], dtype=np.uint8)


def packed_u4_bytes(rows: int, K: int) -> int:
    return ((rows + 31) // 32) * (2 * ((K + 127) // 128)) * FRAGMENT_BYTES


def pack_u4(X: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """X: rows x K matrix with entries in 0..15.  Returns (packed bytes as uint8 vector, int32 sums per row)."""
    X = np.asarray(X)
    if X.ndim != 2 or X.min(initial=0) < 0 or X.max(initial=0) > 15:
        raise ValueError("rows x K matrix with entries in 0..15 expected")
    rows, K = X.shape
    RB, KB = (rows + 31) // 32, 2 * ((K + 127) // 128)
    sums = X.astype(np.int64).sum(axis=1).astype(np.int32)
    out = np.zeros(RB * KB * FRAGMENT_BYTES, dtype=np.uint8)
    for rb in range(RB):
        for kb in range(KB):
            base = (rb * KB + kb) * FRAGMENT_BYTES
            for h in range(2):
                for i in range(32):
                    r = 32 * rb + i
                    string = 0
                    for j in range(32):
                        k = 64 * kb + 32 * h + j
                        v = int(X[r, k]) if (r < rows and k < K) else 0
                        string |= int(CODES[v]) << (6 * j)
                    raw = string.to_bytes(24, "little")
                    slot = 32 * h + i
                    for p in range(3):
                        o = base + p * 512 + slot * 8
                        out[o:o + 8] = np.frombuffer(raw[8 * p:8 * p + 8], dtype=np.uint8)
    return out, sums


def unpack_u4(packed: np.ndarray, rows: int, K: int) -> np.ndarray:
    """Inverse of pack_u4 (decodes through e2m3_value, not through the code table)."""
    packed = np.asarray(packed, dtype=np.uint8)
    RB, KB = (rows + 31) // 32, 2 * ((K + 127) // 128)
    if packed.size != RB * KB * FRAGMENT_BYTES:
        raise ValueError("size mismatch")
    X = np.zeros((rows, K), dtype=np.uint8)
    for r in range(rows):
        rb, i = divmod(r, 32)
        for k in range(K):
            kb, rem = divmod(k, 64)
            h, j = divmod(rem, 32)
            base = (rb * KB + kb) * FRAGMENT_BYTES
            slot = 32 * h + i
            raw = b"".join(bytes(packed[base + p * 512 + slot * 8: base + p * 512 + slot * 8 + 8]) for p in range(3))
            code = (int.from_bytes(raw, "little") >> (6 * j)) & 63
            X[r, k] = int(round(2.0 * e2m3_value(code)))
    return X
