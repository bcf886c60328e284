"""The structured-sparse weight operand (Section VI, "Sparsity"): fpq_pack_weights_sparse against the oracle's 2-of-4
pruning rule code for code, and fpq_gemm_sparse / fpq_conv2d_sparse against the oracle's dense layer on the pruned
codes at the layer tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, check_close, dev, gpu_pack

pytestmark = pytest.mark.gpu
E4M3, E2M1 = synth.E4M3, synth.E2M1


def gpu_pack_sparse(w, fw, h=None, scale=None):
    w_t = dev(w)
    N, Cin = w.shape[0], w.shape[1]
    kh, kw = (w.shape[2], w.shape[3]) if w.ndim == 4 else (1, 1)
    size = B.fpq_packed_sparse_size(N, Cin, kh, kw, fw)
    packed = torch.full((size + 64,), 0xEE, dtype=torch.uint8, device=DEV)
    sw = torch.empty(N, dtype=torch.float32, device=DEV)
    codes = torch.full((w.size,), 0xEE, dtype=torch.uint8, device=DEV)
    dropped = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    B.fpq_pack_weights_sparse(w_t, fw, None if scale is None else dev(scale), None if h is None else dev(h), packed[:size], sw,
                              codes, dropped)
    torch.cuda.synchronize()
    assert np.all(packed[size:].cpu().numpy() == 0xEE), "written beyond the packed buffer"
    return packed[:size], sw, codes.cpu().numpy().reshape(w.shape), int(dropped.item())


PACK_CASES = [((320, 320), E4M3), ((96, 40), E2M1), ((7, 6), E2M1), ((33, 130), E4M3), ((48, 32, 3, 3), E2M1),
              ((20, 6, 3, 3), E4M3), ((64, 64, 1, 1), E2M1), ((10, 20, 5, 5), E2M1)]


@pytest.mark.parametrize("shape,fw", PACK_CASES)
def test_pruned_codes_scales_and_dropped_count_equal_the_oracle(shape, fw):
    w = synth.weights(shape, 4000 + shape[0])
    h = synth.rounding_mask(shape, 4750 + shape[0]) if fw is E2M1 else None
    wq, sw = oracle.pack_weights(w, fw, h)
    want, lost = oracle.prune_2of4_fast(wq, fw)
    _, sw_t, codes, dropped = gpu_pack_sparse(w, fw, h)
    assert np.array_equal(sw_t.cpu().numpy(), sw)
    assert np.array_equal(codes, want), int((codes != want).sum())
    assert dropped == lost
    if w.size <= 4096:
        assert np.array_equal(oracle.prune_2of4(wq, fw)[0], want)


LINEAR = [(5, 48, 3), (77, 768, 320), (130, 128, 65), (256, 320, 320), (300, 2880, 96), (4096, 640, 640), (2048, 1280, 1280)]


@pytest.mark.parametrize("M,K,N", LINEAR)
@pytest.mark.parametrize("fw", [E4M3, E2M1])
@pytest.mark.parametrize("xkind", [B.FPQ_X_CODES, B.FPQ_X_FP32_DYNAMIC])
def test_sparse_linear_layer(M, K, N, fw, xkind):
    fx = E4M3
    x = synth.activations((M, K), 4100 + M)
    w = synth.weights((N, K), 4600 + N)
    h = synth.rounding_mask((N, K), 4850 + N) if fw is E2M1 else None
    bias = np.linspace(-0.5, 0.5, N).astype(np.float32)
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    pruned, lost = oracle.prune_2of4_fast(wq, fw)
    Y, T = oracle.gemm(xq, fx, sx, pruned, fw, sw, bias)
    packed, sw_t, codes, dropped = gpu_pack_sparse(w, fw, h)
    assert np.array_equal(codes, pruned) and dropped == lost
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(max(256, B.fpq_gemm_workspace_size(M, N, K, xkind)), dtype=torch.uint8, device=DEV)
    if xkind == B.FPQ_X_CODES:
        B.fpq_gemm_sparse(dev(xq), 0, fx, sx, None, packed, fw, sw_t, dev(bias), y, M, N, K, ws)
    else:
        B.fpq_gemm_sparse(dev(x), xkind, fx, 0.0, None, packed, fw, sw_t, dev(bias), y, M, N, K, ws)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert not np.isnan(yh).any()
    check_close(yh, Y, T, what="sparse linear %s" % ((M, K, N),))
    if fw is E4M3 and M == 256:
        # E4M3 weights of a Gaussian layer are rarely zero: pruning changes the layer, and the result must be that of the
        # pruned codes, not of the dense ones
        Yd, _ = oracle.gemm(xq, fx, sx, wq, fw, sw, bias)
        assert lost > 0 and np.abs(Yd - Y).max() > 100 * (1e-5 * T + 1e-6).max()


CONV = [(1, 16, 8, 8, 32, 3, 1, 1), (2, 4, 9, 7, 5, 3, 1, 1), (1, 20, 6, 6, 33, 3, 2, 1), (2, 32, 5, 5, 64, 1, 1, 0),
        (1, 48, 12, 10, 130, 3, 1, 0), (1, 320, 16, 16, 96, 3, 1, 1), (2, 40, 8, 8, 40, 5, 1, 2), (8, 320, 32, 32, 320, 3, 1, 1)]


@pytest.mark.parametrize("case", CONV)
@pytest.mark.parametrize("fw", [E4M3, E2M1])
def test_sparse_convolution(case, fw):
    Bn, Cin, H, W, Cout, k, stride, pad = case
    fx = E4M3
    x = synth.activations((Bn, Cin, H, W), 4200 + Cin)
    w = synth.weights((Cout, Cin, k, k), 4700 + Cout)
    h = synth.rounding_mask(w.shape, 4950 + Cout) if fw is E2M1 else None
    bias = np.linspace(-0.5, 0.5, Cout).astype(np.float32)
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    pruned, lost = oracle.prune_2of4_fast(wq, fw)
    big = Bn * H * W * Cout * Cin * k * k > 2e9
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    pos = np.unique(np.random.default_rng(1).integers(0, Bn * Ho * Wo, 300)) if big else None
    Y, T = oracle.conv2d(xq, fx, sx, pruned, fw, sw, bias, stride=stride, pad=pad, pix=pos)
    packed, sw_t, codes, dropped = gpu_pack_sparse(w, fw, h)
    assert np.array_equal(codes, pruned) and dropped == lost
    y = torch.full((Bn, Cout, Ho * Wo), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(B.fpq_conv2d_workspace_size(Bn, Cin, H, W, Cout, k, k, stride, pad, 1), dtype=torch.uint8, device=DEV)
    B.fpq_conv2d_sparse(dev(x), 1, fx, sx, None, packed, fw, sw_t, dev(bias), y, Bn, Cin, H, W, Cout, k, k, stride, pad, ws)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert not np.isnan(yh).any()
    got = yh[pos // (Ho * Wo), :, pos % (Ho * Wo)] if big else yh.reshape(Y.shape)
    check_close(got, Y, T, what="sparse conv %s" % (case,))


def test_weights_that_are_2_of_4_sparse_already_give_the_dense_layer_exactly():
    """Small integers with two zeros in every group of four: nothing is dropped, and every product and sum is an exact
    integer, so the sparse layer, the dense layer and the oracle agree with zero tolerance."""
    fx, fw = E4M3, E2M1
    rng = np.random.default_rng(6)
    M, K, N = 130, 384, 72
    x = rng.choice(np.array([0, 1, 2, 3, 4, 5, 6, 7, 8, -1, -2, -3, -4, -6, -8], dtype=np.float32), (M, K))
    w = rng.choice(np.array([1, 2, 3, 4, 6, -1, -2, -3, -4, -6], dtype=np.float32), (N, K))
    zero = np.argsort(rng.random((N, K // 4, 4)), axis=2)[:, :, :2]
    wg = w.reshape(N, K // 4, 4)
    np.put_along_axis(wg, zero, 0.0, axis=2)
    w = wg.reshape(N, K)
    sc = np.ones(N, dtype=np.float32)
    xq = oracle.quantize(x, fx, 1.0)
    packed, sw_t, codes, dropped = gpu_pack_sparse(w, fw, None, sc)
    assert dropped == 0
    assert np.array_equal(oracle.dequantize(codes, fw, 1.0), w)
    y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    B.fpq_gemm_sparse(dev(xq), 0, fx, 1.0, None, packed, fw, sw_t, None, y, M, N, K, None)
    dense_packed, dsw, _ = gpu_pack(w, fw, None, sc)
    yd = torch.empty_like(y)
    B.fpq_gemm(dev(xq), 0, fx, 1.0, None, dense_packed, fw, dsw, None, yd, M, N, K, B.FPQ_ACC_FP32)
    torch.cuda.synchronize()
    want = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.array_equal(y.cpu().numpy().astype(np.float64), want)
    assert torch.equal(y, yd)


def test_sparse_entry_points_reject_what_they_have_no_kernel_for():
    import ctypes as C
    L = B.lib()
    p = C.c_void_p(4096)
    f, e3 = B.fmt(E4M3), B.fmt(synth.E3M4)
    assert L.fpq_gemm_sparse(p, 0, e3, 1.0, None, p, f, p, None, p, 8, 8, 32, None, 0, None) == -8
    assert L.fpq_gemm_sparse(p, 0, f, 1.0, None, p, B.fmt(synth.E3M0), p, None, p, 8, 8, 32, None, 0, None) == -8
    assert L.fpq_gemm_sparse(p, 0, f, 1.0, None, C.c_void_p(4100), f, p, None, p, 8, 8, 32, None, 0, None) == -5
    assert L.fpq_pack_weights_sparse(p, 8, 32, 1, 1, f, None, None, p, 64, p, None, p, None) == -6
    assert B.fpq_packed_sparse_size(320, 320, 1, 1, E4M3) == 256 + 320 * 192 + 320 * 48
    assert B.fpq_packed_sparse_size(320, 320, 3, 3, E2M1) == 256 + 320 * 2944 // 4 + 320 * 2944 // 8
