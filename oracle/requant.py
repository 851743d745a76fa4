"""Activation threshold applied to the integer product.  TEST INFRASTRUCTURE ONLY.

The paper's algorithms end with the integer matrix C (Section III); a BNN / TNN / TBN layer then maps C back to low-bit
activations with per-channel thresholds.  This is that map, written out elementwise, for C of shape (M, N) with one
threshold pair per row i (output channel):

    ternary:  y = -1 if c < lo[i];  +1 if c > hi[i] and not c < lo[i];  0 otherwise
    binary:   y = -1 if c < lo[i];  +1 otherwise

The result is returned as the next layer's feature map, (N, M) int8: one row per column of C (output pixel), channels
along the row.
"""
from __future__ import annotations

import numpy as np


def requantize(C: np.ndarray, lo: np.ndarray, hi: np.ndarray | None, ternary: bool) -> np.ndarray:
    M, N = C.shape
    Y = np.empty((N, M), dtype=np.int8)
    for i in range(M):
        for j in range(N):
            c = int(C[i, j])
            if c < int(lo[i]):
                y = -1
            elif ternary:
                y = 1 if c > int(hi[i]) else 0
            else:
                y = 1
            Y[j, i] = y
    return Y
