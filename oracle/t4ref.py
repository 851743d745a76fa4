"""Reference packer for ternary / binary operands of the 4-bit floating-point matrix-core product.  TEST INFRASTRUCTURE ONLY.

The product is the one the paper defines (C = A B over {-1, 0, +1}, Section II-A and III-A): its oracle is
gemm_oracle.c, unchanged.  This module fixes, bit for bit, the operand format the library's pack_t4 must produce:

  * every value is stored as the 4-bit floating-point code (1 sign, 2 exponent, 1 mantissa bit, exponent bias 1,
    subnormal at exponent 0 -- the "E2M1" element type of the Open Compute microscaling formats) of that value:
    +1, -1 and 0 are all representable; values are mapped by sign like pack_ternary (x > 0 -> +1, x < 0 -> -1);
  * a matrix is packed as `rows` strings along the depth k; rows are padded to a multiple of 32 and the depth to a
    multiple of 128 with the code of 0;
  * a "fragment" is 32 rows x 64 depth positions: 64 slots of 16 bytes, slot 32*h + i holding depth positions
    64*kb + 32*h + j (j = 0..31) of row 32*rb + i, position j in bits 4j .. 4j+3 of the 128-bit little-endian string;
  * fragments are ordered by row block, then depth block: byte offset (rb * KB + kb) * 1024 with KB = 2*ceil(K/128).
"""
from __future__ import annotations

import numpy as np

FRAGMENT_BYTES = 1024


def e2m1_value(code: int) -> float:
    """Value of a 4-bit code: sign s, exponent e (2 bits, bias 1), mantissa m (1 bit)."""
    s, e, m = (code >> 3) & 1, (code >> 1) & 3, code & 1
    mag = (m / 2.0) if e == 0 else (2.0 ** (e - 1)) * (1.0 + m / 2.0)
    return -mag if s else mag


def code_of(v: int) -> int:
    """The code whose value is v, found by search over all 16 codes (the smallest one: +0 rather than -0)."""
    for code in range(16):
        if e2m1_value(code) == float(v):
            return code
    raise ValueError(f"{v} has no 4-bit code")


def packed_t4_bytes(rows: int, K: int) -> int:
    return ((rows + 31) // 32) * (2 * ((K + 127) // 128)) * FRAGMENT_BYTES


def pack_t4(X: np.ndarray) -> np.ndarray:
    """X: rows x K integer matrix; entries are taken by sign.  Returns the packed bytes as a uint8 vector."""
    X = np.asarray(X)
    if X.ndim != 2:
        raise ValueError("rows x K matrix expected")
    rows, K = X.shape
    RB, KB = (rows + 31) // 32, 2 * ((K + 127) // 128)
    out = np.zeros(RB * KB * FRAGMENT_BYTES, dtype=np.uint8)
    codes = {v: code_of(v) for v in (-1, 0, 1)}
    for rb in range(RB):
        for kb in range(KB):
            base = (rb * KB + kb) * FRAGMENT_BYTES
            for h in range(2):
                for i in range(32):
                    r = 32 * rb + i
                    string = 0
                    for j in range(32):
                        k = 64 * kb + 32 * h + j
                        x = int(X[r, k]) if (r < rows and k < K) else 0
                        string |= codes[(x > 0) - (x < 0)] << (4 * j)
                    o = base + (32 * h + i) * 16
                    out[o:o + 16] = np.frombuffer(string.to_bytes(16, "little"), dtype=np.uint8)
    return out


def unpack_t4(packed: np.ndarray, rows: int, K: int) -> np.ndarray:
    """Inverse of pack_t4 on sign-valued matrices (decodes through e2m1_value)."""
    packed = np.asarray(packed, dtype=np.uint8)
    RB, KB = (rows + 31) // 32, 2 * ((K + 127) // 128)
    if packed.size != RB * KB * FRAGMENT_BYTES:
        raise ValueError("size mismatch")
    X = np.zeros((rows, K), dtype=np.int8)
    for r in range(rows):
        rb, i = divmod(r, 32)
        for k in range(K):
            kb, rem = divmod(k, 64)
            h, j = divmod(rem, 32)
            o = (rb * KB + kb) * FRAGMENT_BYTES + (32 * h + i) * 16
            code = (int.from_bytes(bytes(packed[o:o + 16]), "little") >> (4 * j)) & 15
            X[r, k] = int(e2m1_value(code))
    return X
