"""The same-bitwidth integer baseline (Eq. (4)): calibration, quantizer and packed weights bit for bit against the
oracle, and the integer-matrix-instruction layer against the oracle's exact integer sums."""
import numpy as np
import pytest
import torch

from oracle import uniform as U
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, check_close, dev

pytestmark = pytest.mark.gpu


def gpu_calibrate(x_t, bits):
    out = torch.zeros(16, dtype=torch.uint8, device=DEV)
    ws = torch.empty(B.lib().fpq_int_calibrate_workspace_size(x_t.numel()), dtype=torch.uint8, device=DEV)
    B.fpq_int_calibrate(x_t, bits, out, ws)
    torch.cuda.synchronize()
    return out, B.int_params(out)


@pytest.mark.parametrize("n", [1, 5, 4096, 4099, 1310720, 5000001])
@pytest.mark.parametrize("bits", [8, 4])
def test_calibration_and_codes_equal_the_oracle(n, bits):
    x = synth.activations((n + 1,), 300 + n)[1:]                 # 4-byte aligned, not 16
    x_t = dev(synth.activations((n + 1,), 300 + n))[1:]
    pdev, p = gpu_calibrate(x_t, bits)
    s, z = U.params(x, bits)
    assert (p.scale, p.zero_point, p.min, p.max) == (np.float32(s), z, x.min(), x.max())
    codes = torch.full((n + 8,), 0xEE, dtype=torch.uint8, device=DEV)
    B.fpq_int_quantize(x_t, bits, 0.0, 0, pdev, codes[4:])
    torch.cuda.synchronize()
    got = codes.cpu().numpy()
    assert np.array_equal(got[4:4 + n], U.quantize(x, bits, s, z))
    assert np.all(got[:4] == 0xEE) and np.all(got[4 + n:] == 0xEE)
    # host-side parameters, a scale that is no power of two, a zero point outside the code range
    codes2 = torch.empty(n, dtype=torch.uint8, device=DEV)
    B.fpq_int_quantize(x_t, bits, 0.0371, -3, None, codes2)
    torch.cuda.synchronize()
    assert np.array_equal(codes2.cpu().numpy(), U.quantize(x, bits, float(np.float32(0.0371)), -3))


def test_quantizer_edge_values():
    s, z = 0.25, 7
    v = np.array([0.0, -0.0, 0.125, 0.375, -0.125, 0.625, 1e30, -1e30, np.inf, -np.inf, 1e-45, 61.9, 62.0, 62.1, -1.75, -1.8],
                 dtype=np.float32)
    codes = torch.empty(v.size, dtype=torch.uint8, device=DEV)
    B.fpq_int_quantize(dev(v), 8, s, z, None, codes)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), U.quantize(v, 8, s, z))
    _, p = gpu_calibrate(dev(np.full(9, 3.5, dtype=np.float32)), 8)
    assert (p.scale, p.zero_point) == U.params(np.full(9, 3.5, dtype=np.float32), 8)
    _, p0 = gpu_calibrate(torch.empty(0, dtype=torch.float32, device=DEV), 8)
    assert (p0.scale, p0.zero_point, p0.min, p0.max) == (1.0, 0, 0.0, 0.0)


def gpu_int_pack(w, bits):
    N, K = w.shape
    packed = torch.empty(B.fpq_int_packed_size(N, K, bits), dtype=torch.uint8, device=DEV)
    sw = torch.empty(N, dtype=torch.float32, device=DEV)
    zw = torch.empty(N, dtype=torch.int32, device=DEV)
    codes = torch.full((N * K,), 0xEE, dtype=torch.uint8, device=DEV)
    B.fpq_int_pack_weights(dev(w), bits, packed, sw, zw, codes)
    torch.cuda.synchronize()
    return packed, sw, zw, codes.cpu().numpy().reshape(N, K)


SHAPES = [(256, 320, 320), (1, 16, 1), (5, 48, 3), (77, 768, 320), (130, 128, 65), (64, 2880, 96), (200, 1280, 130),
          (4096, 640, 640), (2048, 1280, 1280), (300, 32768, 64)]


@pytest.mark.parametrize("M,K,N", SHAPES)
@pytest.mark.parametrize("wbits", [8, 4])
def test_integer_layer(M, K, N, wbits):
    x = synth.activations((M, K), 600 + M)
    w = synth.weights((N, K), 650 + N)
    bias = np.linspace(-0.4, 0.4, N).astype(np.float32)
    sx, zx = U.params(x, 8)
    xq = U.quantize(x, 8, sx, zx)
    wq, sw, zw = U.pack_weights(w, wbits)
    Y, T = U.gemm(xq, sx, zx, wq, sw, zw, bias)
    packed, sw_t, zw_t, codes = gpu_int_pack(w, wbits)
    assert np.array_equal(codes, wq) and np.array_equal(sw_t.cpu().numpy(), sw) and np.array_equal(zw_t.cpu().numpy(), zw)
    x_t = dev(x)
    pdev, p = gpu_calibrate(x_t, 8)
    xc = torch.empty(M * K, dtype=torch.uint8, device=DEV)
    B.fpq_int_quantize(x_t, 8, 0.0, 0, pdev, xc)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(max(256, B.fpq_int_gemm_workspace_size(M)), dtype=torch.uint8, device=DEV)
    B.fpq_int_gemm(xc, 0.0, 0, pdev, packed, wbits, sw_t, zw_t, dev(bias), y, M, N, K, ws)
    torch.cuda.synchronize()
    assert np.array_equal(xc.cpu().numpy().reshape(M, K), xq)
    yh = y.cpu().numpy()
    assert not np.isnan(yh).any()
    check_close(yh, Y, T, what="integer layer %s W%d" % ((M, K, N), wbits))
    # the sums are exact integers: the result is the oracle's integer times one fp32 scale, to the last few bits
    I = (xq.astype(np.int64) - zx) @ (wq.astype(np.int64) - zw.astype(np.int64)[:, None]).T
    want = I.astype(np.float64) * (float(np.float32(sx)) * sw.astype(np.float64))[None, :] + bias.astype(np.float64)[None, :]
    assert np.all(np.abs(yh - want) <= 4e-7 * np.abs(want) + 1e-6 * np.abs(bias)[None, :] + 1e-30)


def test_integer_layer_exact_with_unit_scales_and_all_positive_data():
    """Scales of one and integer data: every output is an integer below 2^24, so the layer must equal the integer matrix
    product exactly; the activations are all positive, which puts their zero point outside the code range."""
    rng = np.random.default_rng(8)
    M, K, N = 130, 255 + 1, 72
    x = rng.integers(3, 259, (M, K)).astype(np.float32)          # min 3, max 258 -> s = 1, z = -3
    x[0, 0], x[0, 1] = 3, 258
    w = rng.integers(-7, 9, (N, K)).astype(np.float32)           # 4 bits: 16 levels, s = 1 when the row spans -7 .. 8
    w[:, 0], w[:, 1] = -7, 8
    sx, zx = U.params(x, 8)
    assert (sx, zx) == (1.0, -3)
    xq = U.quantize(x, 8, sx, zx)
    wq, sw, zw = U.pack_weights(w, 4)
    assert np.all(sw == 1.0) and np.all(zw == 7)
    packed, sw_t, zw_t, codes = gpu_int_pack(w, 4)
    y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    ws = torch.empty(B.fpq_int_gemm_workspace_size(M), dtype=torch.uint8, device=DEV)
    B.fpq_int_gemm(dev(xq), sx, zx, None, packed, 4, sw_t, zw_t, None, y, M, N, K, ws)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64), x.astype(np.float64) @ w.astype(np.float64).T)


def test_integer_entry_points_validate():
    import ctypes as C
    L = B.lib()
    p = C.c_void_p(4096)
    assert L.fpq_int_quantize(p, 16, 6, 1.0, 0, None, p, None) == -2
    assert L.fpq_int_quantize(p, 16, 8, 0.0, 0, None, p, None) == -3
    assert L.fpq_int_quantize(None, 0, 8, 1.0, 0, None, None, None) == 0
    assert L.fpq_int_pack_weights(p, 8, 40000, 8, p, 1 << 30, p, p, None, None) == -4
    assert L.fpq_int_gemm(p, 1.0, 0, None, p, 8, p, p, None, p, 8, 8, 24, p, 1 << 20, None) == -5
    assert L.fpq_int_gemm(p, 1.0, 0, None, p, 8, p, p, None, p, 8, 8, 32, p, 16, None) == -6
    assert L.fpq_int_gemm(p, 1.0, 0, None, p, 8, p, p, None, p, 0, 8, 32, p, 16, None) == 0
    assert B.fpq_int_packed_size(320, 320, 8) == 256 + 320 * 384 + 320 * 4
    assert B.fpq_int_packed_size(320, 320, 4) == 256 + 320 * 192 + 320 * 4
