"""im2col lowering of a 2-D convolution, plain loops.  TEST INFRASTRUCTURE ONLY.

The paper computes convolutions as matrix products (Section I; Section IV-A and eq. (5): the depth of the product is
H_k * W_k * C_in): the feature map is unrolled so that every output pixel becomes one bit string / one column of the
right matrix B whose entries are the input values under the kernel window.  This module writes that definition out:

    B[(ky*KW + kx)*C + c, (b*OH + oy)*OW + ox] = fmap[b, oy*sh + ky - ph, ox*sw + kx - pw, c]     (0 outside the map)

with the feature map in NHWC order and OH = (H + 2*ph - KH)//sh + 1, OW likewise.  The matching left matrix holds one
filter per row with the same (ky, kx, c) depth order.
"""
from __future__ import annotations

import numpy as np


def out_size(H: int, W: int, kh: int, kw: int, sh: int, sw: int, ph: int, pw: int):
    return (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1


def im2col(fmap: np.ndarray, kh: int, kw: int, sh: int = 1, sw: int = 1, ph: int = 0, pw: int = 0) -> np.ndarray:
    """fmap: (batch, H, W, C) int8 -> B: (kh*kw*C, batch*OH*OW) int8, zero padded."""
    nb, H, W, C = fmap.shape
    OH, OW = out_size(H, W, kh, kw, sh, sw, ph, pw)
    B = np.zeros((kh * kw * C, nb * OH * OW), dtype=fmap.dtype)
    for b in range(nb):
        for oy in range(OH):
            for ox in range(OW):
                n = (b * OH + oy) * OW + ox
                for ky in range(kh):
                    iy = oy * sh + ky - ph
                    if iy < 0 or iy >= H:
                        continue
                    for kx in range(kw):
                        ix = ox * sw + kx - pw
                        if ix < 0 or ix >= W:
                            continue
                        k0 = (ky * kw + kx) * C
                        B[k0:k0 + C, n] = fmap[b, iy, ix, :]
    return B


def conv2d_direct(fmap: np.ndarray, filt: np.ndarray, sh: int = 1, sw: int = 1, ph: int = 0, pw: int = 0) -> np.ndarray:
    """Direct definition of the convolution (cross-correlation, as CNN layers use it), int64.
    fmap: (batch, H, W, C), filt: (F, kh, kw, C) -> (batch, OH, OW, F)."""
    nb, H, W, C = fmap.shape
    F, kh, kw, C2 = filt.shape
    assert C == C2
    OH, OW = out_size(H, W, kh, kw, sh, sw, ph, pw)
    padded = np.zeros((nb, H + 2 * ph, W + 2 * pw, C), dtype=np.int64)
    padded[:, ph:ph + H, pw:pw + W, :] = fmap
    out = np.zeros((nb, OH, OW, F), dtype=np.int64)
    f64 = filt.astype(np.int64)
    for oy in range(OH):
        for ox in range(OW):
            win = padded[:, oy * sh:oy * sh + kh, ox * sw:ox * sw + kw, :]           # (nb, kh, kw, C)
            out[:, oy, ox, :] = np.tensordot(win, f64, axes=([1, 2, 3], [1, 2, 3]))
    return out
