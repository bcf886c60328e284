"""Pins of the rounding-learning oracle (Section V-B, Eq. (10)-(14)): CPU only.

The oracle's arithmetic is tied to things other than itself: the already pinned mask quantizer of Eq. (12) at the two
ends of the sigmoid, central finite differences of the loss for the analytic gradient, hand-computed scalar cases and
the closed form of the regulariser."""
import math

import numpy as np
import pytest

import oracle
from oracle import rounding as R
from paper_2408_06995_amd import synth

FORMATS = [synth.E2M1, synth.E4M3, (1, 2, 1, 1.75), (3, 0, 4, 8.0), (2, 1, 2, 3.0)]


def layer(N, K, M, seed, fmt):
    rng = np.random.default_rng(seed)
    W = (rng.normal(0, 0.02, (N, K)) * rng.uniform(0.5, 2, (N, 1))).astype(np.float32)
    sw = (np.abs(W).max(axis=1) / np.float32(fmt[3])).astype(np.float32)
    A = rng.normal(0, 1, (M, K)).astype(np.float32)
    alpha = rng.normal(0, 2, (N, K))
    return W, sw, A, alpha


@pytest.mark.parametrize("fmt", FORMATS)
def test_saturated_sigmoid_reproduces_the_mask_quantizer(fmt):
    """sigmoid(alpha) = 0 / 1 exactly: the soft weight is the dequantized code of Eq. (12) with h = 0 / 1."""
    W, sw, _, _ = layer(7, 33, 1, 3, fmt)
    W[0, :4] = [0.0, -0.0, W[0].max() * 3, -W[0].max() * 3]          # zero and values the clamp catches
    with np.errstate(over="ignore"):
        for h, a in ((0, -800.0), (1, 800.0)):
            Wq, dWq = R.soft_weights(W, sw, np.full(W.shape, a), fmt)
            codes = np.stack([oracle.quantize_mask(W[n], np.full(W.shape[1], h, np.uint8), fmt, sw[n]) for n in range(7)])
            want = oracle.dequantize(codes, fmt) * sw.astype(np.float64)[:, None]
            assert np.array_equal(Wq, want)
            assert np.all(dWq == 0)


@pytest.mark.parametrize("fmt", FORMATS)
def test_gradient_equals_central_finite_differences(fmt):
    W, sw, A, alpha = layer(3, 5, 6, 11, fmt)
    g = R.gradient(W, sw, alpha, A, fmt, reg_weight=0.7)
    num = np.zeros_like(alpha)
    h = 1e-6
    for i in range(alpha.shape[0]):
        for j in range(alpha.shape[1]):
            ap, am = alpha.copy(), alpha.copy()
            ap[i, j] += h
            am[i, j] -= h
            lp, lm = R.loss(W, sw, ap, A, fmt, 0.7), R.loss(W, sw, am, A, fmt, 0.7)
            num[i, j] = ((lp[0] + 0.7 * lp[1]) - (lm[0] + 0.7 * lm[1])) / (2 * h)
    assert np.allclose(g, num, rtol=2e-5, atol=1e-10)


def test_regulariser_closed_forms():
    assert R.regulariser(np.zeros((2, 2)))[0] == 1.0                                      # sigmoid = 0.5
    with np.errstate(over="ignore"):
        assert R.regulariser(np.array([[800.0, -800.0]]))[0] == 0.0                       # sigmoid = 1, 0
    a = math.log(3.0)                                                                     # sigmoid = 0.75
    lam, d = R.regulariser(np.array([[a, -a]]))
    assert lam == pytest.approx(1 - 0.5 ** 20, rel=1e-14)
    # d/da [1 - (2 (s - 0.5))^20] = -20 (2 (s - 0.5))^19 * 2 * s (1 - s) at s = 0.75, divided by the 2 elements
    want = -20 * 0.5 ** 19 * 2 * 0.75 * 0.25 / 2
    assert d[0, 0] == pytest.approx(want, rel=1e-13) and d[0, 1] == pytest.approx(-want, rel=1e-13)


def test_scalar_layer_by_hand():
    """One weight 0.8 on the E2M1 grid (scale 1): neighbours 0.5 and 1.0, step 0.5, floor 1 step."""
    fmt = synth.E2M1
    W, sw, A = np.array([[0.8]], np.float32), np.array([1.0], np.float32), np.array([[2.0]], np.float32)
    a = 0.3
    sg = 1 / (1 + math.exp(-a))
    wq = 0.5 * (1 + sg)
    w = float(np.float32(0.8))
    mse, reg = R.loss(W, sw, np.array([[a]]), A, fmt)
    assert mse == pytest.approx((2 * wq - 2 * w) ** 2, rel=1e-13)
    assert reg == pytest.approx(1 - (2 * (sg - 0.5)) ** 20, rel=1e-13)
    g = R.gradient(W, sw, np.array([[a]]), A, fmt, reg_weight=0.0)
    assert g[0, 0] == pytest.approx(2 * (2 * wq - 2 * w) * 2 * 0.5 * sg * (1 - sg), rel=1e-13)


@pytest.mark.parametrize("fmt", FORMATS)
def test_initial_alpha_starts_from_the_unquantized_weights(fmt):
    W, sw, A, _ = layer(6, 40, 9, 5, fmt)
    a0 = R.init_alpha(W, sw, fmt)
    Wq, _ = R.soft_weights(W, sw, a0, fmt)
    yc, s, fl = R.on_format_axis(W, sw, fmt)
    frac = yc / s - fl
    ok = (frac >= 1e-3) & (frac <= 1 - 1e-3)
    assert ok.mean() > 0.9
    assert np.allclose(Wq[ok], (yc * sw.astype(np.float64)[:, None])[ok], rtol=1e-12, atol=1e-300)
    # and the hard decision of that start is round-to-nearest
    near = oracle.quantize(W[0], fmt, sw[0])
    hard = oracle.quantize_mask(W[0], R.mask(a0)[0], fmt, sw[0])
    differ = near != hard
    assert np.all(np.abs(frac[0][differ] - 0.5) < 1e-9)             # only exact ties may differ (ties-to-even vs >= 0.5)


def test_descent_lowers_the_loss_and_sharpens_the_decisions():
    fmt = synth.E2M1
    W, sw, A, _ = layer(8, 32, 64, 21, fmt)
    alpha = R.init_alpha(W, sw, fmt)
    l0 = R.loss(W, sw, alpha, A, fmt, 0.01)
    # the output error of rounding to nearest, the baseline that learning is meant to beat or match
    for _ in range(300):
        alpha, _, _ = R.step(W, sw, alpha, A, fmt, lr=2000.0, reg_weight=0.01)
    l1 = R.loss(W, sw, alpha, A, fmt, 0.01)
    assert l1[0] + 0.01 * l1[1] < l0[0] + 0.01 * l0[1]
    assert l1[1] < l0[1]


@pytest.mark.parametrize("k,stride,pad", [(3, 1, 1), (3, 2, 1), (1, 1, 0), (5, 1, 2), (3, 1, 0)])
def test_patch_matrix_turns_a_convolution_into_the_linear_layer(k, stride, pad):
    """Against torch's unfold (a library routine) and against the convolution itself: A W^T = conv(x, W)."""
    import torch
    rng = np.random.default_rng(k * 10 + stride)
    x = rng.normal(0, 1, (2, 5, 9, 7))
    w = rng.normal(0, 1, (4, 5, k, k))
    A = R.im2col(x, k, k, stride, pad)
    unf = torch.nn.functional.unfold(torch.from_numpy(x), (k, k), padding=pad, stride=stride)     # [B, C k k, L]
    assert np.array_equal(A, unf.permute(0, 2, 1).reshape(-1, 5 * k * k).numpy())
    y = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=stride, padding=pad).numpy()
    assert np.allclose(A @ w.reshape(4, -1).T, y.transpose(0, 2, 3, 1).reshape(-1, 4), rtol=1e-12, atol=1e-12)
