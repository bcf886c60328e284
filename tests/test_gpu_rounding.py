"""Rounding learning (Section V-B, Eq. (10)-(14)): the HIP step against the double-precision oracle.

Tolerances.  The step is fp32 throughout: the output error R = A (Wq - W)^T is a sum of K products of fp32 values whose
second factor carries the rounding of Wq - W (one ulp of |W|), so |R_gpu - R| <= 1e-5 * sum_k |A_k| (|D_k| + 1e-6 |W_k|);
the losses are sums of non-negative terms (relative 1e-4); the gradient d mse / d Wq is a sum over M rows of products R A
with the error of R carried through, bounded by 2e-5 * (2 / (M N)) sum_m (|R| + err R) |A|, times d Wq / d alpha."""
import numpy as np
import pytest
import torch

import oracle
from oracle import rounding as R
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, dev

pytestmark = pytest.mark.gpu

E2M1, E4M3, E1M2 = synth.E2M1, synth.E4M3, (1, 2, 1, 1.75)


def layer(N, K, M, seed, fmt):
    W = synth.weights((N, K), seed)
    sw = (np.abs(W).max(axis=1) / np.float32(fmt[3])).astype(np.float32)
    A = synth.activations((M, K), seed + 1)
    rng = np.random.default_rng(seed + 2)
    alpha = rng.normal(0, 2, (N, K)).astype(np.float32)
    return W, sw, A, alpha


def gpu_step(W, sw, alpha, A, fmt, lr, regw, want_grad=True):
    N, K = W.shape
    M = A.shape[0]
    al = dev(alpha.copy())
    loss = torch.full((2,), float("nan"), device=DEV)
    grad = torch.full((N, K), float("nan"), device=DEV) if want_grad else None
    ws = torch.empty(B.fpq_rl_workspace_size(M, N, K), dtype=torch.uint8, device=DEV)
    B.fpq_rl_step(dev(W), dev(sw), fmt, al, dev(A), lr, regw, loss, grad, ws)
    torch.cuda.synchronize()
    return al.cpu().numpy(), loss.cpu().numpy(), None if grad is None else grad.cpu().numpy()


# N, K, M: below one tile, ragged in every direction, several 64-tiles, the 128-tile kernel, a deep contraction over M
SHAPES = [(3, 5, 6), (33, 70, 45), (130, 96, 200), (320, 320, 256), (640, 1280, 2048), (64, 48, 5000)]


@pytest.mark.parametrize("N,K,M", SHAPES)
@pytest.mark.parametrize("fmt", [E2M1, E4M3, E1M2])
def test_step_against_oracle(N, K, M, fmt):
    check_step(N, K, M, fmt, 9000 + N)


@pytest.mark.parametrize("i", range(24))
def test_step_on_random_shapes(i):
    """Shapes drawn at random: every combination of ragged tiles of the two fp32 contractions and of their K slices."""
    rng = np.random.default_rng(9500 + i)
    N, K, M = int(rng.integers(1, 400)), int(rng.integers(1, 500)), int(rng.integers(1, 3000))
    fmt = [E2M1, E4M3, E1M2, (3, 0, 4, 8.0)][i % 4]
    print("case", i, (N, K, M), fmt, flush=True)
    check_step(N, K, M, fmt, 9600 + i)


def check_step(N, K, M, fmt, seed):
    W, sw, A, alpha = layer(N, K, M, seed, fmt)
    lr, regw = 50.0, 0.3
    a1, loss, grad = gpu_step(W, sw, alpha, A, fmt, lr, regw)
    mse, reg = R.loss(W, sw, alpha, A, fmt, regw)
    assert loss[0] == pytest.approx(mse, rel=1e-4)
    assert loss[1] == pytest.approx(reg, rel=1e-4)
    # gradient: bound from the module docstring
    Wq, dWq = R.soft_weights(W, sw, alpha, fmt)
    A64, W64 = A.astype(np.float64), W.astype(np.float64)
    D = Wq - W64
    Rm = A64 @ D.T
    errR = 1e-5 * (np.abs(A64) @ (np.abs(D) + 1e-6 * np.abs(W64)).T)
    errG = 2e-5 * (2.0 / Rm.size) * ((np.abs(Rm) + errR).T @ np.abs(A64)) + (2.0 / Rm.size) * (errR.T @ np.abs(A64))
    g = R.gradient(W, sw, alpha, A, fmt, regw)
    # plus the fp32 evaluation of the two terms themselves (they can cancel in g)
    Gm = (2.0 / Rm.size) * (Rm.T @ A64)
    tol = errG * np.abs(dWq) + 1e-5 * (np.abs(Gm * dWq) + regw * np.abs(R.regulariser(alpha)[1])) + 1e-12
    bad = np.abs(grad - g) > tol
    assert not bad.any(), (int(bad.sum()), float((np.abs(grad - g) / tol).max()))
    # the update is alpha - lr * (the gradient the kernel reports), in fp32
    assert np.allclose(a1, alpha - np.float32(lr) * grad, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("fmt", [E2M1, E4M3, (3, 0, 4, 8.0)])
def test_init_alpha_and_mask(fmt):
    N, K = 37, 129
    W = synth.weights((N, K), 9500)
    W[0, :3] = [0.0, -0.0, W[1].max() * 5]
    sw = (np.abs(W[1:]).max() / np.float32(fmt[3]) * np.ones(N)).astype(np.float32)
    al = torch.full((N, K), float("nan"), device=DEV)
    B.fpq_rl_init_alpha(dev(W), dev(sw), fmt, al)
    mk = torch.full((N * K,), 7, dtype=torch.uint8, device=DEV)
    B.fpq_rl_mask(al, mk)
    torch.cuda.synchronize()
    a_gpu = al.cpu().numpy()
    a0 = R.init_alpha(W, sw, fmt)
    assert np.allclose(a_gpu, a0, rtol=1e-5, atol=1e-5)
    assert np.array_equal(mk.cpu().numpy().reshape(N, K), (a_gpu >= 0).astype(np.uint8))
    agree = mk.cpu().numpy().reshape(N, K) == R.mask(a0)
    assert agree.mean() > 0.999                                # only alphas within rounding of 0 may differ
    assert np.all(np.abs(a0[~agree]) < 1e-5)


def test_learning_run_follows_the_oracle_and_feeds_pack_weights():
    """40 steps from the initial alpha on a small layer: the loss curve follows the oracle's, and the learned mask goes
    through fpq_pack_weights like any other mask."""
    fmt = E2M1
    N, K, M = 64, 96, 512
    W, sw, A, _ = layer(N, K, M, 9700, fmt)
    lr, regw = 3000.0, 0.01
    al = torch.empty((N, K), device=DEV)
    Wd, swd, Ad = dev(W), dev(sw), dev(A)
    B.fpq_rl_init_alpha(Wd, swd, fmt, al)
    loss = torch.zeros(2, device=DEV)
    ws = torch.empty(B.fpq_rl_workspace_size(M, N, K), dtype=torch.uint8, device=DEV)
    a_or = R.init_alpha(W, sw, fmt)
    curve_gpu, curve_or = [], []
    for _ in range(40):
        B.fpq_rl_step(Wd, swd, fmt, al, Ad, lr, regw, loss, None, ws)
        curve_gpu.append(loss.cpu().numpy().copy())
        a_or, mse, reg = R.step(W, sw, a_or, A, fmt, lr, regw)
        curve_or.append((mse, reg))
    curve_gpu, curve_or = np.array(curve_gpu), np.array(curve_or)
    assert np.allclose(curve_gpu[:, 1], curve_or[:, 1], rtol=2e-3)
    assert np.allclose(curve_gpu[1:, 0], curve_or[1:, 0], rtol=2e-2)        # the first entry is ~0: start = unquantized weights
    assert curve_gpu[-1, 1] < curve_gpu[0, 1]                               # decisions sharpen
    mk = torch.empty(N * K, dtype=torch.uint8, device=DEV)
    B.fpq_rl_mask(al, mk)
    torch.cuda.synchronize()
    h = mk.cpu().numpy().reshape(N, K)
    from gpu_util import gpu_pack
    _, _, codes = gpu_pack(W, fmt, h, scale_np=sw)
    wq, _ = oracle.pack_weights(W, fmt, h, sw)
    assert np.array_equal(codes, wq)
    # the learned rounding is not worse at the layer output than round-to-nearest (what learning is for)
    A64 = A.astype(np.float64)
    def out_err(cq):
        return float(np.mean((A64 @ (oracle.dequantize(cq, fmt) * sw.astype(np.float64)[:, None] - W.astype(np.float64)).T) ** 2))
    near, _ = oracle.pack_weights(W, fmt, None, sw)
    assert out_err(wq) <= out_err(near) * 1.05


@pytest.mark.parametrize("case", [(2, 5, 9, 7, 3, 1, 1), (1, 16, 12, 12, 3, 2, 1), (3, 4, 6, 6, 1, 1, 0), (1, 3, 11, 8, 5, 1, 2)])
def test_patch_matrix_exact_and_conv_step(case):
    """The patch matrix is a copy (exact); a rounding-learning step of a convolution = the linear step on it."""
    Bn, C, H, W, k, stride, pad = case
    x = synth.activations((Bn, C, H, W), 9800 + C)
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    M, K = Bn * Ho * Wo, C * k * k
    a = torch.full((M, K), float("nan"), device=DEV)
    B.fpq_rl_im2col(dev(x), k, k, stride, pad, a)
    torch.cuda.synchronize()
    A = R.im2col(x, k, k, stride, pad)
    assert np.array_equal(a.cpu().numpy().astype(np.float64), A)
    fmt = E2M1
    N = 6
    Wt = synth.weights((N, C, k, k), 9850).reshape(N, K)
    sw = (np.abs(Wt).max(axis=1) / np.float32(fmt[3])).astype(np.float32)
    alpha = R.init_alpha(Wt, sw, fmt).astype(np.float32)
    al = dev(alpha.copy())
    loss = torch.zeros(2, device=DEV)
    grad = torch.zeros((N, K), device=DEV)
    ws = torch.empty(B.fpq_rl_workspace_size(M, N, K), dtype=torch.uint8, device=DEV)
    B.fpq_rl_step(dev(Wt), dev(sw), fmt, al, a, 10.0, 0.1, loss, grad, ws)
    torch.cuda.synchronize()
    mse, reg = R.loss(Wt, sw, alpha, A.astype(np.float32), fmt, 0.1)
    g = R.gradient(Wt, sw, alpha, A.astype(np.float32), fmt, 0.1)
    assert loss.cpu().numpy()[0] == pytest.approx(mse, rel=1e-3, abs=1e-12)
    assert loss.cpu().numpy()[1] == pytest.approx(reg, rel=1e-4)
    assert np.allclose(grad.cpu().numpy(), g, rtol=1e-3, atol=1e-6 * np.abs(g).max() + 1e-12)


def test_argument_checks():
    import ctypes as C
    L = B.lib()
    t = torch.zeros(1024, device=DEV)
    P = C.c_void_p(t.data_ptr())
    f = B.fmt(E2M1)
    assert L.fpq_rl_step(P, P, 4, 4, f, P, P, 4, 0.1, 0.1, P, None, P, 16, None) == -6
    assert L.fpq_rl_step(P, P, 4, 4, f, P, P, 0, 0.1, 0.1, P, None, P, 1 << 20, None) == -4
    assert L.fpq_rl_step(P, P, 4, 4, f, None, P, 4, 0.1, 0.1, P, None, P, 1 << 20, None) == -1
    assert L.fpq_rl_step(P, P, 4, 4, f, P, P, 4, float("nan"), 0.1, P, None, P, 1 << 20, None) == -3
    assert L.fpq_rl_step(P, P, 4, 4, B.fmt((2, 1, 1, 5.0)), P, P, 4, 0.1, 0.1, P, None, P, 1 << 20, None) == -2
    assert L.fpq_rl_init_alpha(P, None, 4, 4, f, P, None) == -1
    assert B.fpq_rl_workspace_size(0, 4, 4) == 0
