"""Pins for the oracle's binary convolution (CPU only).

Sec. 3.1 of the paper maps a convolution layer to a GEMM with M = filters,
N = batch x output pixels, K = kernel_h x kernel_w x input channels.  The oracle's
im2col + GEMM form is pinned from three independent sides: its own direct nested-loop
form, torch's conv2d on the sign of the explicitly zero-padded image (library routine),
and closed forms on constant inputs that fix the padding rule (padded taps count as +1).
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

RNG = np.random.default_rng(77)

CASES = [
    # N, C, H, W, O, k, s, p
    (1, 1, 1, 1, 1, 1, 1, 0),
    (2, 3, 5, 5, 4, 3, 1, 1),
    (1, 20, 8, 5, 3, 3, 2, 1),
    (2, 64, 5, 8, 5, 3, 1, 1),
    (1, 65, 8, 8, 2, 5, 2, 2),
    (1, 3, 8, 8, 2, 5, 1, 0),
    (1, 2, 2, 2, 3, 3, 1, 1),
    (2, 4, 7, 7, 3, 1, 2, 0),
    (1, 5, 9, 9, 2, 7, 1, 3),
]


def torch_ref(x, w, s, p):
    xp = F.pad(torch.from_numpy(x).double(), (p, p, p, p), value=0.0)
    sx = torch.where(xp >= 0, 1.0, -1.0).double()
    sw = torch.where(torch.from_numpy(w) >= 0, 1.0, -1.0).double()
    return F.conv2d(sx, sw, stride=s, padding=0).numpy().astype(np.int32)


@pytest.mark.parametrize("N,C,H,W,O,k,s,p", CASES)
def test_conv_three_ways(N, C, H, W, O, k, s, p):
    x = RNG.standard_normal((N, C, H, W)).astype(np.float32)
    w = RNG.standard_normal((O, C, k, k)).astype(np.float32)
    oi, of = oracle.binary_conv2d(x, w, s, p)
    np.testing.assert_array_equal(oi, oracle.binary_conv2d_direct(x, w, s, p))
    np.testing.assert_array_equal(oi, torch_ref(x, w, s, p))
    np.testing.assert_array_equal(of, oi.astype(np.float32))
    Ho, Wo = oracle.conv_out_hw(H, W, k, k, s, p)
    assert oi.shape == (N, O, Ho, Wo)


def test_conv_is_gemm_of_im2col():
    """M = filters, N = batch x pixels, K = kh x kw x C (Sec. 3.1)."""
    N, C, H, W, O, k, s, p = 2, 6, 6, 7, 5, 3, 1, 1
    x = RNG.standard_normal((N, C, H, W)).astype(np.float32)
    w = RNG.standard_normal((O, C, k, k)).astype(np.float32)
    col = oracle.im2col(x, k, k, s, p)
    assert col.shape == (N * 6 * 7, k * k * C)
    # zero padding present in the float im2col, and the unfold agrees with torch's
    ref = F.unfold(torch.from_numpy(x), k, padding=p, stride=s)  # [N, C*k*k, L]
    np.testing.assert_array_equal(col.reshape(N, 42, -1), ref.permute(0, 2, 1).numpy())
    g, _ = oracle.binary_fc(w.reshape(O, -1), col)  # [O, N*L]
    oi, _ = oracle.binary_conv2d(x, w, s, p)
    np.testing.assert_array_equal(oi, g.reshape(O, N, 6, 7).transpose(1, 0, 2, 3))


def test_conv_padding_closed_forms():
    """All-(+1) input and weights give K everywhere, borders included; an all-(-1) input
    gives -K inside and -K + 2*C*(padded taps) on the border (padded taps are +1)."""
    C, H, W, O = 5, 6, 6, 2
    K = 9 * C
    wp = np.ones((O, C, 3, 3), dtype=np.float32)
    oi, _ = oracle.binary_conv2d(np.ones((1, C, H, W), dtype=np.float32), wp, 1, 1)
    assert (oi == K).all()
    oi, _ = oracle.binary_conv2d(-np.ones((1, C, H, W), dtype=np.float32), wp, 1, 1)
    for h, w in itertools.product(range(H), range(W)):
        taps_out = sum(1 for dh in (-1, 0, 1) for dw in (-1, 0, 1)
                       if not (0 <= h + dh < H and 0 <= w + dw < W))
        assert (oi[0, :, h, w] == -K + 2 * C * taps_out).all()
    assert oi[0, 0, 2, 2] == -K and oi[0, 0, 0, 0] == -K + 2 * C * 5 and oi[0, 0, 0, 3] == -K + 2 * C * 3


def test_conv_alpha_per_output_channel():
    x = RNG.standard_normal((2, 3, 4, 4)).astype(np.float32)
    w = RNG.standard_normal((3, 3, 3, 3)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    oi, of = oracle.binary_conv2d(x, w, 1, 1, alpha)
    np.testing.assert_array_equal(of, alpha[None, :, None, None] * oi.astype(np.float32))


def test_conv_single_weight_flip_moves_output_by_two():
    """A transposed or mis-indexed weight tensor cannot pass: flip one weight, exactly the
    outputs of that filter that see the tap change, by +-2."""
    x = np.abs(RNG.standard_normal((1, 2, 4, 4))).astype(np.float32) + 0.1  # all +1
    w = np.ones((2, 2, 3, 3), dtype=np.float32)
    base, _ = oracle.binary_conv2d(x, w, 1, 0)
    w[1, 0, 2, 0] = -1.0
    got, _ = oracle.binary_conv2d(x, w, 1, 0)
    np.testing.assert_array_equal(got[0, 0], base[0, 0])
    np.testing.assert_array_equal(got[0, 1], base[0, 1] - 2)


def test_batchnorm_folds_into_a_threshold():
    """The block of Sec. 2 ends QConvolution -> BatchNorm, and the next block starts with the
    sign: sign(gamma * (v - mean) / sigma + beta) is the compare v >= mean - beta * sigma / gamma
    for gamma > 0 (negated operands for gamma < 0).  Checked on every value a layer of K = 18
    can produce (v = alpha * dot, dot in -K .. K step 2), in exact rational arithmetic away from
    the tie, so that the threshold form the bit-output entry points take is the BatchNorm."""
    from fractions import Fraction as F
    K = 18
    for alpha, gamma, beta, mean, sigma in [(F(1, 2), F(3, 2), F(-1, 4), F(5, 8), F(7, 4)),
                                            (F(3, 4), F(-2), F(1, 3), F(-1, 2), F(5, 4)),
                                            (F(1), F(1, 7), F(0), F(0), F(1))]:
        thr = mean - beta * sigma / gamma
        for dot in range(-K, K + 1, 2):
            v = alpha * dot
            bn = gamma * (v - mean) / sigma + beta
            if gamma > 0:
                assert (bn >= 0) == (v >= thr)
            elif bn != 0:  # gamma < 0: alpha and thr negated (the tie itself flips sides)
                assert (bn >= 0) == (-alpha * dot >= -thr)
