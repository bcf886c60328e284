"""Every launch configuration the planner of the layer calls can produce -- kernel (small register-staged tiles,
128 x 160 tiles, 256 x 160 tiles, the at-most-16-rows kernel) x number of K slices -- compared with the oracle:
linear layers and convolutions, E4M3 and E2M1 weights, fp32 results and results as codes.  Each case first asserts,
through the library's read-only plan query, that its shape still takes the configuration it is meant to cover."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, check_close, dev, gpu_pack
from test_gpu_codes_out import check_codes, out_scale

pytestmark = pytest.mark.gpu

E4M3, E2M1 = synth.E4M3, synth.E2M1
SMALL, T256, T128, ROWS16 = B.FPQ_KERNEL_SMALL_TILE, B.FPQ_KERNEL_256x160, B.FPQ_KERNEL_128x160, B.FPQ_KERNEL_ROWS16


def rows_to_check(M, seed, tile=128, n_tiles=12, n_random=24):
    """First and last row of the first, the last and some random tiles, plus random rows."""
    rng = np.random.default_rng(seed)
    nt = (M + tile - 1) // tile
    tiles = np.unique(np.concatenate([[0, nt - 1], rng.integers(0, nt, n_tiles)]))
    rows = np.concatenate([tiles * tile, np.minimum(tiles * tile + tile - 1, M - 1), rng.integers(0, M, n_random)])
    return np.unique(rows)


# (M, K, N, kernel, K slices): the planner's outcomes.  The 256-row tile takes 2 .. 5 slices when its tile grid
# alone would fill between a fifth and three quarters of the compute units and K is deep enough; the 128-row tile is
# sliced to about one work item per compute unit.
LINEAR_PLANS = [
    (8, 1280, 1280, ROWS16, 1),
    (616, 768, 320, SMALL, 1),
    (4096, 640, 640, T128, 1),
    (3072, 2048, 2560, T256, 1),
    (2048, 8192, 2080, T256, 2),
    (1280, 12288, 2720, T256, 3),
    (1024, 16384, 2560, T256, 4),
    (768, 20480, 2560, T256, 5),
    (8192, 2560, 640, T128, 1),
    (2048, 5120, 1280, T128, 2),
    (1408, 4096, 1280, T128, 3),
    (1024, 4096, 1280, T128, 4),
    (512, 5120, 1280, T128, 5),
    (512, 8192, 1600, T128, 7),
    (512, 11520, 1280, T128, 8),
    (128, 32768, 1280, T128, 32),
]


@pytest.mark.parametrize("M,K,N,kernel,slices", LINEAR_PLANS,
                         ids=["M%d_K%d_N%d_k%d_s%d" % c for c in LINEAR_PLANS])
def test_linear_every_plan(M, K, N, kernel, slices):
    assert B.fpq_gemm_plan(M, N, K) == (kernel, slices), "this shape no longer takes the plan it is here to cover"
    want_ws = slices * M * N * 4 if slices > 1 else 0
    assert B.fpq_gemm_workspace_size(M, N, K, 0) == (want_ws + 255) // 256 * 256
    fx = E4M3
    x = synth.activations((M, K), 7000 + M)
    w = synth.weights((N, K), 7500 + N)
    h = synth.rounding_mask((N, K), 7750 + N)
    bias = np.linspace(-0.4, 0.4, N).astype(np.float32)
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    xq_t = dev(xq)
    pos = np.arange(M) if M <= 1024 else rows_to_check(M, M + K)
    ws = torch.empty(max(256, B.fpq_gemm_workspace_size(M, N, K, 0)), dtype=torch.uint8, device=DEV)
    for fw, mask in ((E4M3, None), (E2M1, h)):
        wq, sw = oracle.pack_weights(w, fw, mask)
        Y, T = oracle.gemm(xq, fx, sx, wq, fw, sw, bias, rows=pos)
        packed, sw_t, _ = gpu_pack(w, fw, mask, want_codes=False)
        what = "linear %s %s" % ((M, K, N, kernel, slices), "E4M3" if fw is E4M3 else "E2M1")
        # fp32 result
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        B.fpq_gemm(xq_t, 0, fx, sx, None, packed, fw, sw_t, dev(bias), y, M, N, K, B.FPQ_ACC_FP32, ws)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        assert not np.isnan(yh).any(), "unwritten outputs: " + what
        check_close(yh[pos], Y, T, what=what)
        # result as codes for a following layer (E4M3, static scale); the at-most-16-rows kernel has no such form
        # of its own, the call then takes the small-tile kernel
        sy = out_scale(Y, E4M3)
        Np = B.fpq_padded_channels(N)
        yq = torch.full((M * Np,), 0xEE, dtype=torch.uint8, device=DEV)
        B.fpq_gemm_codes_out(xq_t, 0, fx, sx, None, packed, fw, sw_t, dev(bias), E4M3, sy, None, yq, M, N, K,
                             B.FPQ_ACC_FP32, ws)
        torch.cuda.synchronize()
        got = yq.cpu().numpy().reshape(M, Np)
        miss = check_codes(got[pos], Y, T, E4M3, sy, 1e-5, what + " codes out")
        assert miss < 0.002


# (B, Cin, H, W, Cout, k, stride, kernel, K slices)
CONV_PLANS = [
    (2, 64, 24, 24, 320, 3, 1, SMALL, 1),
    (8, 320, 64, 64, 320, 1, 1, T128, 1),
    (8, 320, 32, 32, 320, 3, 1, T128, 2),
    (8, 320, 64, 64, 320, 3, 1, T256, 1),
    (8, 960, 32, 32, 640, 3, 1, T256, 2),
    (8, 1920, 16, 16, 1280, 3, 1, T256, 4),
    (8, 1280, 16, 16, 1280, 3, 1, T128, 4),
    (8, 1280, 8, 8, 1280, 3, 1, T128, 8),
    (8, 640, 32, 32, 640, 3, 2, T128, 4),
]


@pytest.mark.parametrize("case", CONV_PLANS, ids=["B%d_C%d_%dx%d_N%d_k%d_s%d_k%d_s%d" % c for c in CONV_PLANS])
def test_conv_every_plan(case):
    Bn, Cin, H, W, Cout, k, stride, kernel, slices = case
    pad = k // 2
    assert B.fpq_conv2d_plan(Bn, Cin, H, W, Cout, k, k, stride, pad) == (kernel, slices), \
        "this shape no longer takes the plan it is here to cover"
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    M = Bn * Ho * Wo
    fx = E4M3
    x = synth.activations((Bn, Cin, H, W), 8000 + Cin + H)
    w = synth.weights((Cout, Cin, k, k), 8500 + Cout)
    h = synth.rounding_mask(w.shape, 8750 + Cout)
    bias = np.linspace(-0.4, 0.4, Cout).astype(np.float32)
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    x_t = dev(x)
    pos = rows_to_check(M, M + Cin)
    ws = torch.empty(B.fpq_conv2d_workspace_size(Bn, Cin, H, W, Cout, k, k, stride, pad, 1), dtype=torch.uint8, device=DEV)
    for fw, mask in ((E4M3, None), (E2M1, h)):
        wq, sw = oracle.pack_weights(w, fw, mask)
        Y, T = oracle.conv2d(xq, fx, sx, wq, fw, sw, bias, stride=stride, pad=pad, pix=pos)
        packed, sw_t, _ = gpu_pack(w, fw, mask, want_codes=False)
        what = "conv %s %s" % (case, "E4M3" if fw is E4M3 else "E2M1")
        y = torch.full((Bn, Cout, Ho * Wo), float("nan"), dtype=torch.float32, device=DEV)
        B.fpq_conv2d(x_t, 1, fx, sx, None, packed, fw, sw_t, dev(bias), y, Bn, Cin, H, W, Cout, k, k, stride, pad,
                     B.FPQ_ACC_FP32, ws)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        assert not np.isnan(yh).any(), "unwritten outputs: " + what
        check_close(yh[pos // (Ho * Wo), :, pos % (Ho * Wo)], Y, T, what=what)
        sy = out_scale(Y, E4M3)
        Np = B.fpq_padded_channels(Cout)
        yq = torch.full((M * Np,), 0xEE, dtype=torch.uint8, device=DEV)
        B.fpq_conv2d_codes_out(x_t, 1, fx, sx, None, packed, fw, sw_t, dev(bias), E4M3, sy, None, yq, Bn, Cin, H, W, Cout,
                               k, k, stride, pad, B.FPQ_ACC_FP32, ws)
        torch.cuda.synchronize()
        got = yq.cpu().numpy().reshape(M, Np)
        miss = check_codes(got[pos], Y, T, E4M3, sy, 1e-5, what + " codes out")
        assert miss < 0.002
