"""Pins for the im2col oracle (no GPU): against the direct convolution definition, against scipy's correlate, and on
hand-checkable cases."""
import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import im2col as oi
from oracle import oracle


def _rand_ternary(rng, shape):
    return rng.integers(-1, 2, size=shape).astype(np.int8)


@pytest.mark.parametrize("geom", [(1, 5, 6, 3, 3, 3, 1, 1, 1, 1), (2, 7, 5, 4, 3, 2, 2, 1, 0, 1),
                                  (1, 4, 4, 2, 1, 1, 1, 1, 0, 0), (2, 6, 6, 5, 2, 2, 2, 2, 1, 0)])
def test_im2col_gemm_equals_direct_convolution(geom):
    nb, H, W, C, kh, kw, sh, sw, ph, pw = geom
    rng = np.random.default_rng(sum(geom))
    fmap = _rand_ternary(rng, (nb, H, W, C))
    filt = _rand_ternary(rng, (7, kh, kw, C))
    B = oi.im2col(fmap, kh, kw, sh, sw, ph, pw)
    A = np.ascontiguousarray(filt.reshape(7, kh * kw * C))
    OH, OW = oi.out_size(H, W, kh, kw, sh, sw, ph, pw)
    Cmat = oracle.gemm(A, np.ascontiguousarray(B))                               # F x (nb*OH*OW)
    got = Cmat.reshape(7, nb, OH, OW).transpose(1, 2, 3, 0)
    assert np.array_equal(got, oi.conv2d_direct(fmap, filt, sh, sw, ph, pw))


def test_direct_convolution_against_scipy():
    """Single channel, stride 1: the direct definition is scipy's 2-D cross-correlation of the zero-padded map."""
    rng = np.random.default_rng(3)
    fmap = _rand_ternary(rng, (1, 8, 9, 1))
    filt = _rand_ternary(rng, (1, 3, 3, 1))
    want = correlate2d(np.pad(fmap[0, :, :, 0].astype(np.int64), 1), filt[0, :, :, 0].astype(np.int64), mode="valid")
    assert np.array_equal(oi.conv2d_direct(fmap, filt, 1, 1, 1, 1)[0, :, :, 0], want)


def test_im2col_hand_case():
    """2x2 map, one channel, 2x2 window, no padding: one output pixel whose column is the map in row-major order;
    with padding 1 there are 9 pixels and the centre one sees the whole map."""
    fmap = np.array([[[[1], [-1]], [[0], [1]]]], dtype=np.int8)                   # (1, 2, 2, 1)
    B = oi.im2col(fmap, 2, 2)
    assert B.shape == (4, 1) and B[:, 0].tolist() == [1, -1, 0, 1]
    Bp = oi.im2col(fmap, 2, 2, 1, 1, 1, 1)
    assert Bp.shape == (4, 9)
    assert Bp[:, 0].tolist() == [0, 0, 0, 1]                                      # top-left window: only its last tap hits (0,0)
    assert Bp[:, 4].tolist() == [1, -1, 0, 1]
    assert Bp[:, 8].tolist() == [1, 0, 0, 0]


def test_channel_is_fastest_depth_index():
    fmap = np.arange(2 * 2 * 3, dtype=np.int8).reshape(1, 2, 2, 3) - 5
    B = oi.im2col(fmap, 1, 2)                                                      # window 1x2, two output pixels
    assert B[:, 0].tolist() == fmap[0, 0, 0, :].tolist() + fmap[0, 0, 1, :].tolist()
    assert B[:, 1].tolist() == fmap[0, 1, 0, :].tolist() + fmap[0, 1, 1, :].tolist()
