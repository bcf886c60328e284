"""Seeded random sweep of layer shapes, formats, accumulate modes and input forms against the oracle: ragged M, N and
K, widths on and off the large-tile kernels' multiple of 160, kernel sizes 1 / 3 / 5, strides 1 - 3, paddings up to
the kernel's half width plus one, with and without bias, codes / fp32 / dynamic-scale inputs, results as fp32 or as
codes.  Every case is compared in full; the case is printed before its launch."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, check_close, dev, gpu_pack

pytestmark = pytest.mark.gpu

E4M3, E5M2, E2M1 = synth.E4M3, synth.E5M2, synth.E2M1
HW_PAIRS = [(E4M3, E4M3), (E4M3, E2M1), (E4M3, E5M2), (E5M2, E4M3)]
SOFT_PAIRS = [(synth.E3M4, synth.E3M0), (synth.E2M5, (4, 3, 7, 480.0)), ((4, 3, 9, 112.0), (2, 1, 2, 3.0)),
              (E4M3, synth.E1M2)]
REL_FP8_MFMA = 7 * 2.0 ** -13


def resolved(f):
    e, m, b, c = f
    return (e, m, b, c if c else oracle.format_max(e, m, b))


def pick_case(rng, kind):
    hw = rng.random() < 0.6
    fx, fw = (HW_PAIRS if hw else SOFT_PAIRS)[rng.integers(0, 4)]
    acc = B.FPQ_ACC_FP8_MFMA if hw and rng.random() < 0.3 else B.FPQ_ACC_FP32
    wide = rng.random() < 0.45
    N = int(160 * rng.integers(1, 5)) if wide else int(rng.integers(1, 400))
    c = {"fx": resolved(fx), "fw": resolved(fw), "acc": acc, "N": N, "bias": bool(rng.random() < 0.6),
         "mask": bool(rng.random() < 0.6), "xin": int(rng.integers(0, 3)), "codes_out": bool(rng.random() < 0.25)}
    if kind == "linear":
        c["M"] = int(rng.choice([1, 2, 7, 16, 17, 63, 64, 65, 127, 129, 255, 300, 513, 700, 1100]))
        c["K"] = int(rng.choice([16, 32, 48, 112, 128, 144, 320, 400, 768, 1296, 2576]))
        if c["xin"] and rng.random() < 0.5:
            c["K"] = int(rng.integers(1, 700))          # fp32 input takes any K
    else:
        c["B"] = int(rng.integers(1, 4))
        c["Cin"] = int(rng.choice([1, 3, 4, 16, 20, 33, 48, 64, 130, 320]))
        c["k"] = int(rng.choice([1, 3, 3, 3, 5]))
        c["stride"] = int(rng.choice([1, 1, 1, 2, 3]))
        c["pad"] = int(rng.integers(0, c["k"] // 2 + 2))
        c["H"] = int(rng.integers(max(1, c["k"] - 2 * c["pad"]), 24))
        c["W"] = int(rng.integers(max(1, c["k"] - 2 * c["pad"]), 24))
    return c


def check_codes_out(yq, Y, T, fy, sy, rel):
    """The code of every output must be the quantizer's code of some value within the layer's tolerance of the
    oracle's result (the quantizer is monotone), and equal the oracle's own code where that leaves no choice."""
    lo, hi = oracle.requantize_bounds(Y, T, fy, sy, rel, 1e-6)
    vlo, vhi, vg = (oracle.dequantize(c, fy) for c in (lo, hi, yq))
    bad = (vg < vlo) | (vg > vhi)
    assert not bad.any(), "%d of %d codes outside the tolerance interval" % (int(bad.sum()), bad.size)
    same = lo == hi
    assert np.array_equal(yq[same], lo[same])


@pytest.mark.parametrize("i", range(72))
def test_random_linear(i):
    rng = np.random.default_rng(7000 + i)
    c = pick_case(rng, "linear")
    print("case", i, c, flush=True)
    M, K, N, fx, fw = c["M"], c["K"], c["N"], c["fx"], c["fw"]
    x = synth.activations((M, K), 7100 + i)
    w = synth.weights((N, K), 7200 + i)
    h = synth.rounding_mask((N, K), 7300 + i) if c["mask"] else None
    bias = np.linspace(-1, 1, N).astype(np.float32) if c["bias"] else None
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    if c["xin"] == 1:
        sx = float(np.float32(sx * 1.37))               # a static scale that clips
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    packed, sw_t, _ = gpu_pack(w, fw, h, want_codes=False)
    xin = c["xin"]
    xarg = dev(x) if xin else dev(xq)
    ws = torch.empty(max(256, B.fpq_gemm_workspace_size(M, N, K, xin)), dtype=torch.uint8, device=DEV)
    bias_t = None if bias is None else dev(bias)
    Y, T = oracle.gemm(xq, fx, sx, wq, fw, sw, bias)
    rel = REL_FP8_MFMA if c["acc"] else 1e-5
    if c["codes_out"]:
        fy = resolved(E4M3)
        sy = oracle.scale_from_absmax(float(np.abs(Y).max()), fy[3])
        Np = B.fpq_padded_channels(N)
        yq = torch.full((M, Np), 0xA5, dtype=torch.uint8, device=DEV)
        B.fpq_gemm_codes_out(xarg, xin, fx, sx, None, packed, fw, sw_t, bias_t, fy, sy, None, yq, M, N, K, c["acc"], ws)
        torch.cuda.synchronize()
        got = yq.cpu().numpy()
        assert np.all(got[:, N:] == 0)
        check_codes_out(got[:, :N], Y, T, fy, sy, rel)
    else:
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        B.fpq_gemm(xarg, xin, fx, sx, None, packed, fw, sw_t, bias_t, y, M, N, K, c["acc"], ws)
        torch.cuda.synchronize()
        check_close(y.cpu().numpy(), Y, T, rel=rel, what=str(c))


@pytest.mark.parametrize("i", range(56))
def test_random_conv(i):
    rng = np.random.default_rng(8000 + i)
    c = pick_case(rng, "conv")
    print("case", i, c, flush=True)
    Bn, Cin, H, W, Cout, k, stride, pad, fx, fw = (c["B"], c["Cin"], c["H"], c["W"], c["N"], c["k"], c["stride"],
                                                    c["pad"], c["fx"], c["fw"])
    x = synth.activations((Bn, Cin, H, W), 8100 + i)
    w = synth.weights((Cout, Cin, k, k), 8200 + i)
    h = synth.rounding_mask(w.shape, 8300 + i) if c["mask"] else None
    bias = np.linspace(-0.5, 0.5, Cout).astype(np.float32) if c["bias"] else None
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    if c["xin"] == 1:
        sx = float(np.float32(sx * 1.37))
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    packed, sw_t, _ = gpu_pack(w, fw, h, want_codes=False)
    xin = c["xin"]
    if xin:
        xarg = dev(x)
    else:
        Cp = B.fpq_padded_channels(Cin)
        xarg = torch.empty(Bn * H * W * Cp, dtype=torch.uint8, device=DEV)
        B.fpq_quantize_nhwc(dev(x), fx, sx, None, xarg)
    ws = torch.empty(max(256, B.fpq_conv2d_workspace_size(Bn, Cin, H, W, Cout, k, k, stride, pad, xin)), dtype=torch.uint8,
                     device=DEV)
    bias_t = None if bias is None else dev(bias)
    Y, T = oracle.conv2d(xq, fx, sx, wq, fw, sw, bias, stride=stride, pad=pad)
    Ho, Wo = Y.shape[2], Y.shape[3]
    rel = REL_FP8_MFMA if c["acc"] else 1e-5
    if c["codes_out"]:
        fy = resolved(E4M3)
        sy = oracle.scale_from_absmax(float(np.abs(Y).max()), fy[3])
        Np = B.fpq_padded_channels(Cout)
        yq = torch.full((Bn * Ho * Wo, Np), 0xA5, dtype=torch.uint8, device=DEV)
        B.fpq_conv2d_codes_out(xarg, xin, fx, sx, None, packed, fw, sw_t, bias_t, fy, sy, None, yq, Bn, Cin, H, W, Cout, k, k,
                               stride, pad, c["acc"], ws)
        torch.cuda.synchronize()
        got = yq.cpu().numpy().reshape(Bn, Ho, Wo, Np)
        assert np.all(got[..., Cout:] == 0)
        nhwc = lambda a: np.ascontiguousarray(a.transpose(0, 2, 3, 1))
        check_codes_out(got[..., :Cout], nhwc(Y), nhwc(T), fy, sy, rel)
    else:
        y = torch.full((Bn, Cout, Ho, Wo), float("nan"), dtype=torch.float32, device=DEV)
        B.fpq_conv2d(xarg, xin, fx, sx, None, packed, fw, sw_t, bias_t, y, Bn, Cin, H, W, Cout, k, k, stride, pad, c["acc"], ws)
        torch.cuda.synchronize()
        check_close(y.cpu().numpy(), Y, T, rel=rel, what=str(c))


ALL_FORMATS = [E4M3, E5M2, E2M1, synth.E1M2, synth.E3M4, synth.E2M5, synth.E3M0, (4, 3, 7, 480.0), (4, 3, 9, 112.0),
               (5, 2, 15, 0.0), (2, 1, 2, 3.0), (3, 2, 3, 28.0), (1, 6, 1, 0.0), (4, 3, -3, 0.0), (2, 3, 1, 0.875)]


@pytest.mark.parametrize("i", range(40))
def test_random_pack_weights(i):
    """Weight codes and scales, bit for bit: random shape and format, with / without mask, computed or given scales."""
    rng = np.random.default_rng(8500 + i)
    f = resolved(ALL_FORMATS[int(rng.integers(0, len(ALL_FORMATS)))])
    k = int(rng.choice([1, 1, 3, 5]))
    shape = (int(rng.integers(1, 200)), int(rng.integers(1, 300)), k, k)
    print("case", i, shape, f, flush=True)
    w = synth.weights(shape, 8600 + i)
    w.reshape(-1)[::int(rng.integers(2, 50))] = 0.0
    if rng.random() < 0.3:
        w[int(rng.integers(0, shape[0]))] = 0.0                       # an all-zero output channel
    h = synth.rounding_mask(shape, 8700 + i) if rng.random() < 0.6 else None
    sc = rng.uniform(0.001, 0.05, shape[0]).astype(np.float32) if rng.random() < 0.4 else None
    want_codes, want_sw = oracle.pack_weights(w, f, h, sc)
    _, sw, codes = gpu_pack(w, f, h, sc)
    assert np.array_equal(sw.cpu().numpy(), want_sw)
    assert np.array_equal(codes, want_codes), int((codes != want_codes).sum())


@pytest.mark.parametrize("i", range(32))
def test_random_quantize_nhwc(i):
    """Channels-last activation codes with channel padding, bit for bit, static and device scale."""
    rng = np.random.default_rng(8800 + i)
    f = resolved([E4M3, E5M2, synth.E3M4, synth.E2M5, (4, 3, 7, 480.0)][int(rng.integers(0, 5))])
    shape = (int(rng.integers(1, 5)), int(rng.integers(1, 200)), int(rng.integers(1, 40)), int(rng.integers(1, 40)))
    print("case", i, shape, f, flush=True)
    x = synth.activations(shape, 8900 + i)
    sx = float(np.float32(oracle.scale_from_absmax(oracle.absmax(x), f[3]) * rng.uniform(0.5, 1.5)))
    Bn, Cc, H, W = shape
    Cp = B.fpq_padded_channels(Cc)
    codes = torch.full((Bn * H * W * Cp + 16,), 0xEE, dtype=torch.uint8, device=DEV)
    if i & 1:
        B.fpq_quantize_nhwc(dev(x), f, 0.0, dev(np.array([sx], dtype=np.float32)), codes)
    else:
        B.fpq_quantize_nhwc(dev(x), f, sx, None, codes)
    torch.cuda.synchronize()
    got = codes.cpu().numpy()
    assert np.all(got[Bn * H * W * Cp:] == 0xEE)
    got = got[:Bn * H * W * Cp].reshape(Bn, H, W, Cp)
    assert np.array_equal(got[..., :Cc], oracle.quantize(x, f, sx).transpose(0, 2, 3, 1))
    assert np.all(got[..., Cc:] == 0)
