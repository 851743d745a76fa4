"""GPU parity for the packed-domain im2col and the convolution it feeds (bit-exact against the CPU oracles)."""
import sys

import numpy as np
import pytest
import torch

from oracle import bitref, oracle
from oracle import im2col as oi
from paper_2205_09120_amd import binding as lb
from paper_2205_09120_amd import synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def words(t):
    return t.cpu().numpy().view(np.uint64)


GEOMS = [  # batch, H, W, C, kh, kw, sh, sw, ph, pw
    (1, 5, 6, 64, 3, 3, 1, 1, 1, 1),
    (2, 7, 5, 128, 3, 2, 2, 1, 0, 1),
    (3, 4, 4, 192, 1, 1, 1, 1, 0, 0),
    (2, 9, 8, 64, 5, 3, 2, 3, 2, 1),
    (1, 3, 3, 64, 3, 3, 1, 1, 0, 0),
    (2, 6, 6, 256, 2, 2, 2, 2, 1, 0),
]


def _fmap(kind, geom, seed):
    nb, H, W, C = geom[:4]
    X, _ = synth.make_custom(kind, nb * H * W, 1, C, seed)              # (pixels, C) with the kind's value set
    return X.reshape(nb, H, W, C)


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("ternary", [True, False])
def test_im2col_packed_matches_reference(geom, ternary):
    nb, H, W, C, kh, kw, sh, sw, ph, pw = geom
    say(f"im2col_packed geom={geom} ternary={ternary}")
    fmap = _fmap("tnn" if ternary else "bnn", geom, seed=sum(geom))
    d = torch.from_numpy(fmap).cuda()
    pack = lb.pack_ternary if ternary else lb.pack_binary
    Fp = pack(d, nb * H * W, C, C, 1)
    Bp = lb.im2col_packed(Fp, 2 if ternary else 1, nb, H, W, C, kh, kw, sh, sw, ph, pw)
    torch.cuda.synchronize()
    B = oi.im2col(fmap, kh, kw, sh, sw, ph, pw)                          # (K, N) int8, zero padded
    Bt = np.ascontiguousarray(B.T)
    if ternary:
        want = bitref.pack_ternary(Bt)
    else:
        # zero padding has no binary code; the library writes bit 0 (= +1) there, which is what the reference
        # packer produces for a zero entry (x < 0 is false)
        want = bitref.pack_binary(Bt)
    assert np.array_equal(words(Bp), want.reshape(-1))


@pytest.mark.parametrize("geom", GEOMS[:4])
def test_convolution_through_im2col_packed(geom):
    """Filters (ternary) x feature map (ternary): gemm_tnn on the gathered operand equals the direct convolution."""
    nb, H, W, C, kh, kw, sh, sw, ph, pw = geom
    say(f"conv via im2col_packed + gemm_tnn geom={geom}")
    F = 37
    fmap = _fmap("tnn", geom, seed=7 + sum(geom))
    filt, _ = synth.make_custom("tnn", F, 1, kh * kw * C, seed=11)
    OH, OW = oi.out_size(H, W, kh, kw, sh, sw, ph, pw)
    N, K = nb * OH * OW, kh * kw * C
    Ap = lb.pack_a("tnn", torch.from_numpy(filt).cuda())
    Fp = lb.pack_ternary(torch.from_numpy(fmap).cuda(), nb * H * W, C, C, 1)
    Bp = lb.im2col_packed(Fp, 2, nb, H, W, C, kh, kw, sh, sw, ph, pw)
    Cm = lb.gemm_tnn(F, N, K, Ap, Bp)
    torch.cuda.synchronize()
    got = Cm.cpu().numpy().reshape(F, nb, OH, OW).transpose(1, 2, 3, 0)
    want = oi.conv2d_direct(fmap, filt.reshape(F, kh, kw, C), sh, sw, ph, pw)
    assert np.array_equal(got, want)


def test_im2col_packed_headline_geometry():
    """Batch 16 of 56x56x512 maps, 3x3 window, padding 1: the geometry behind the 4608 x 50176 benchmark operand.
    Checked on sampled output strings (every tap, including padded borders) against the reference."""
    nb, H, W, C, kh, kw = 16, 56, 56, 512, 3, 3
    say("im2col_packed headline geometry 16x56x56x512, 3x3, pad 1")
    rng = np.random.default_rng(5)
    fmap = synth.draw_ternary(rng, (nb * H * W, C), 0.5).reshape(nb, H, W, C)
    Fp = lb.pack_ternary(torch.from_numpy(fmap).cuda(), nb * H * W, C, C, 1)
    Bp = lb.im2col_packed(Fp, 2, nb, H, W, C, kh, kw, 1, 1, 1, 1)
    torch.cuda.synchronize()
    got = words(Bp).reshape(nb * H * W, kh * kw * (C // 64), 2)
    Fref = bitref.pack_ternary(fmap.reshape(-1, C)).reshape(nb, H, W, C // 64, 2)
    pix = [(0, 0, 0), (0, 0, 55), (0, 55, 0), (15, 55, 55), (3, 17, 0), (7, 0, 31), (9, 28, 28)]
    pix += [tuple(int(v) for v in p) for p in np.stack([rng.integers(0, nb, 200), rng.integers(0, H, 200),
                                                         rng.integers(0, W, 200)], axis=1)]
    for (b, oy, ox) in pix:
        n = (b * H + oy) * W + ox
        for ky in range(kh):
            for kx in range(kw):
                iy, ix = oy + ky - 1, ox + kx - 1
                blk = got[n, (ky * kw + kx) * (C // 64):(ky * kw + kx + 1) * (C // 64)]
                if 0 <= iy < H and 0 <= ix < W:
                    assert np.array_equal(blk, Fref[b, iy, ix]), (b, oy, ox, ky, kx)
                else:
                    assert not blk.any(), (b, oy, ox, ky, kx)


@pytest.mark.parametrize("out_planes", [2, 1])
def test_two_convolution_layers_stay_packed(out_planes):
    """Layer 1 (3x3, pad 1) with the activation threshold fused into the product, layer 2 (3x3, stride 2) on its
    packed output: the feature map between the layers exists only as packed words.  Oracle: direct convolution,
    threshold by definition, direct convolution."""
    from oracle import requant
    nb, H, W, C0, F1, F2 = 2, 12, 10, 64, 128, 40
    ternary_mid = out_planes == 2
    say(f"two conv layers on packed data, middle feature map {'ternary' if ternary_mid else 'binary'}")
    fmap = _fmap("tnn", (nb, H, W, C0), seed=21)
    w1, _ = synth.make_custom("tnn", F1, 1, 9 * C0, seed=22)
    w2, _ = synth.make_custom("tnn", F2, 1, 9 * F1, seed=23)
    rng = np.random.default_rng(24)
    lo = rng.integers(-12, -2, size=F1).astype(np.int32)
    hi = rng.integers(2, 12, size=F1).astype(np.int32)
    # ---- oracle
    c1 = oi.conv2d_direct(fmap, w1.reshape(F1, 3, 3, C0), 1, 1, 1, 1)            # (nb, H, W, F1)
    C1 = np.ascontiguousarray(c1.reshape(nb * H * W, F1).T).astype(np.int32)     # (F1, pixels) as the product yields it
    Y = requant.requantize(C1, lo, hi if ternary_mid else None, ternary_mid)     # (pixels, F1) int8
    mid = Y.reshape(nb, H, W, F1)
    OH, OW = oi.out_size(H, W, 3, 3, 2, 2, 0, 0)
    want = oi.conv2d_direct(mid, w2.reshape(F2, 3, 3, F1), 2, 2, 0, 0)           # (nb, OH, OW, F2)
    # ---- library: pack -> gather -> product + threshold -> gather -> product
    Fp = lb.pack_ternary(torch.from_numpy(fmap).cuda(), nb * H * W, C0, C0, 1)
    B1 = lb.im2col_packed(Fp, 2, nb, H, W, C0, 3, 3, 1, 1, 1, 1)
    A1 = lb.pack_a("tnn", torch.from_numpy(w1).cuda())
    Mid = lb.gemm_requant("tnn", out_planes, F1, nb * H * W, 9 * C0, A1, B1, torch.from_numpy(lo).cuda(),
                          torch.from_numpy(hi).cuda() if ternary_mid else None)
    torch.cuda.synchronize()
    ref_mid = (bitref.pack_ternary(Y) if ternary_mid else bitref.pack_binary(Y)).reshape(-1)
    assert np.array_equal(words(Mid), ref_mid)
    B2 = lb.im2col_packed(Mid, out_planes, nb, H, W, F1, 3, 3, 2, 2, 0, 0)
    kind2 = "tnn" if ternary_mid else "tbn"                                      # ternary filters x binary map
    A2 = lb.pack_a(kind2, torch.from_numpy(w2).cuda())
    C2 = lb.gemm(kind2, F2, nb * OH * OW, 9 * F1, A2, B2)
    torch.cuda.synchronize()
    got = C2.cpu().numpy().reshape(F2, nb, OH, OW).transpose(1, 2, 3, 0)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ convolution as an implicit product (conv_gemm)

CONV_GEOMS = GEOMS + [
    (2, 20, 17, 64, 3, 3, 1, 1, 1, 1),      # 680 output pixels: several V tiles and a ragged last one
    (1, 33, 31, 128, 3, 3, 2, 2, 1, 1),     # stride 2 with padding
    (3, 11, 13, 64, 1, 5, 1, 2, 0, 2),      # flat window, channel words < words per stage
    (1, 40, 40, 320, 3, 3, 1, 1, 1, 1),     # 5 channel words: taps do not align with the staging chunks
]


@pytest.mark.parametrize("geom", CONV_GEOMS)
def test_conv_gemm_ternary_matches_direct_convolution(geom):
    """conv_gemm (ternary filters x ternary map) against the definition of the convolution, for every tile variant."""
    nb, H, W, C, kh, kw, sh, sw, ph, pw = geom
    F = 70
    fmap = _fmap("tnn", geom, seed=31 + sum(geom))
    filt, _ = synth.make_custom("tnn", F, 1, kh * kw * C, seed=33)
    OH, OW = oi.out_size(H, W, kh, kw, sh, sw, ph, pw)
    N = nb * OH * OW
    want = oi.conv2d_direct(fmap, filt.reshape(F, kh, kw, C), sh, sw, ph, pw)
    Ap = lb.pack_a("tnn", torch.from_numpy(filt).cuda())
    Fp = lb.pack_ternary(torch.from_numpy(fmap).cuda(), nb * H * W, C, C, 1)
    try:
        for v in list(range(lb.lb_num_variants("tnn"))) + [-1]:
            say(f"conv_gemm tnn geom={geom} variant={v}")
            lb.lb_set_variant("tnn", v)
            Cm = torch.full((F, N + 2), -3, dtype=torch.int32, device="cuda")
            lb.conv_gemm("tnn", F, Ap, Fp, nb, H, W, C, kh, kw, sh, sw, ph, pw, Cm, N + 2)
            torch.cuda.synchronize()
            got = Cm.cpu().numpy()
            assert np.all(got[:, N:] == -3)
            assert np.array_equal(got[:, :N].reshape(F, nb, OH, OW).transpose(1, 2, 3, 0), want), v
    finally:
        lb.lb_set_variant("tnn", -1)


@pytest.mark.parametrize("geom", CONV_GEOMS[:8])
def test_conv_gemm_binary_pads_with_plus_one(geom):
    """Binary filters x binary map: a binary map has no code for 0, positions outside the map count as +1.  Checked
    against the direct convolution of a map that is padded with +1 explicitly (and has no padding of its own left)."""
    nb, H, W, C, kh, kw, sh, sw, ph, pw = geom
    say(f"conv_gemm bnn geom={geom}")
    F = 33
    fmap = _fmap("bnn", geom, seed=41 + sum(geom))
    filt, _ = synth.make_custom("bnn", F, 1, kh * kw * C, seed=43)
    padded = np.ones((nb, H + 2 * ph, W + 2 * pw, C), dtype=np.int8)
    padded[:, ph:ph + H, pw:pw + W, :] = fmap
    want = oi.conv2d_direct(padded, filt.reshape(F, kh, kw, C), sh, sw, 0, 0)
    OH, OW = oi.out_size(H, W, kh, kw, sh, sw, ph, pw)
    Ap = lb.pack_a("bnn", torch.from_numpy(filt).cuda())
    Fp = lb.pack_binary(torch.from_numpy(fmap).cuda(), nb * H * W, C, C, 1)
    Cm = lb.conv_gemm("bnn", F, Ap, Fp, nb, H, W, C, kh, kw, sh, sw, ph, pw)
    torch.cuda.synchronize()
    got = Cm.cpu().numpy().reshape(F, nb, OH, OW).transpose(1, 2, 3, 0)
    assert np.array_equal(got, want)
    # the two-step lowering writes the same values
    Bp = lb.im2col_packed(Fp, 1, nb, H, W, C, kh, kw, sh, sw, ph, pw)
    C2 = lb.gemm_bnn(F, nb * OH * OW, kh * kw * C, Ap, Bp)
    torch.cuda.synchronize()
    assert torch.equal(C2, Cm)


def test_conv_gemm_headline_geometry():
    """Batch 16 of 56x56x512 maps, 1024 filters of 3x3x512, padding 1 -- the layer behind the benchmark's 1024 x 50176
    x 4608 product -- at full size in the default launch configuration: sampled outputs recomputed by the oracle from
    the unrolled definition, and every output equal to the product on the materialised operand."""
    nb, H, W, C, kh, kw, F = 16, 56, 56, 512, 3, 3, 1024
    say("conv_gemm headline geometry 16x56x56x512, 1024 filters 3x3, pad 1")
    rng = np.random.default_rng(6)
    fmap = synth.draw_ternary(rng, (nb * H * W, C), 0.5).reshape(nb, H, W, C)
    filt = synth.draw_ternary(rng, (F, kh * kw * C), 0.5)
    Ap = lb.pack_a("tnn", torch.from_numpy(filt).cuda())
    Fp = lb.pack_ternary(torch.from_numpy(fmap).cuda(), nb * H * W, C, C, 1)
    N, K = nb * H * W, kh * kw * C
    Cm = lb.conv_gemm("tnn", F, Ap, Fp, nb, H, W, C, kh, kw, 1, 1, 1, 1)
    Bp = lb.im2col_packed(Fp, 2, nb, H, W, C, kh, kw, 1, 1, 1, 1)
    C2 = lb.gemm_tnn(F, N, K, Ap, Bp)
    torch.cuda.synchronize()
    assert torch.equal(Cm, C2)
    # sampled pixels (corners, edges, interior) x all filters: columns of the unrolled operand built by the definition
    pix = [(0, 0, 0), (0, 0, 55), (0, 55, 0), (15, 55, 55), (3, 17, 0), (7, 0, 31), (9, 28, 28)]
    pix += [tuple(int(v) for v in p) for p in np.stack([rng.integers(0, nb, 40), rng.integers(0, H, 40),
                                                        rng.integers(0, W, 40)], axis=1)]
    cols = np.zeros((K, len(pix)), dtype=np.int8)
    for j, (b, oy, ox) in enumerate(pix):
        for ky in range(kh):
            for kx in range(kw):
                iy, ix = oy + ky - 1, ox + kx - 1
                if 0 <= iy < H and 0 <= ix < W:
                    cols[(ky * kw + kx) * C:(ky * kw + kx + 1) * C, j] = fmap[b, iy, ix]
    want = oracle.gemm(filt, cols)                                   # (F, samples)
    idx = torch.tensor([(b * H + oy) * W + ox for (b, oy, ox) in pix], device="cuda")
    got = Cm[:, idx].cpu().numpy()
    assert np.array_equal(got, want)


def test_conv_gemm_argument_rules():
    say("conv_gemm: ternary-binary operands are refused, empty problems are no-ops")
    Fp = torch.zeros(64, dtype=torch.int64, device="cuda")
    Ap = torch.zeros(64, dtype=torch.int64, device="cuda")
    with pytest.raises(lb.LowbitError) as e:
        lb.conv_gemm("tbn", 4, Ap, Fp, 1, 2, 2, 64, 1, 1)
    assert e.value.status == lb.LB_EUNSUPPORTED
    lb.conv_gemm("tnn", 0, None, None, 1, 2, 2, 64, 1, 1)
    lb.conv_gemm("tnn", 4, None, None, 0, 2, 2, 64, 1, 1)
    lb.conv_gemm("tnn", 4, None, None, 1, 2, 2, 64, 3, 3)            # window larger than the unpadded map
    with pytest.raises(lb.LowbitError) as e:
        lb.conv_gemm("tnn", 4, Ap, Fp, 1, 2, 2, 100, 1, 1)
    assert e.value.status == lb.LB_EUNSUPPORTED                      # channels not a multiple of 64
