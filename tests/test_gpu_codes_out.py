"""Layers whose result leaves as codes for the next quantized layer (fpq_gemm_codes_out / fpq_conv2d_codes_out).

The epilogue quantizes the kernel's own fp32 value v, which equals the oracle's double-precision Y only within the
layer tolerance; the quantizer is monotone, so the check is: the value of every GPU code lies between the values of
Q(Y - tol) and Q(Y + tol), and (what is unique) equals the oracle's code wherever those two agree.  Cases whose sums
are exact in fp32 are compared code for code."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, dev, gpu_pack, oracle_linear_inputs

pytestmark = pytest.mark.gpu

REL_FP8_MFMA = 7 * 2.0 ** -13
E4M3, E2M1, E3M4, E5M2 = synth.E4M3, synth.E2M1, synth.E3M4, synth.E5M2


def check_codes(got, Y, T, fy, sy, rel, what):
    """got: uint8 [M, Np]; Y, T: float64 [M, N]."""
    M, N = Y.shape
    assert got.shape[0] == M and got.shape[1] == B.fpq_padded_channels(N)
    assert np.all(got[:, N:] == 0), "%s: padding columns must hold code 0" % what
    g = got[:, :N]
    lo, hi = oracle.requantize_bounds(Y, T, fy, sy, rel, 1e-6)
    vlo, vhi, vg = (oracle.dequantize(c, fy) for c in (lo, hi, g))
    bad = (vg < vlo) | (vg > vhi)
    assert not bad.any(), "%s: %d of %d codes outside the tolerance interval" % (what, int(bad.sum()), bad.size)
    same = lo == hi
    assert np.array_equal(g[same], lo[same]), what
    # the kernel's fp32 sums are far closer to the exact ones than the tolerance allows, so next to all codes equal
    # those of the exactly rounded result
    return float((g != oracle.requantize(Y, fy, sy)).mean())


def out_scale(Y, fy):
    return float(np.float32(np.abs(Y).max() / fy[3] * 0.8))    # some outputs clip


def gpu_linear_codes(xq, sx, fx, packed, fw, sw_t, bias, fy, sy, M, N, K, acc, sy_on_device=False):
    Np = B.fpq_padded_channels(N)
    buf = torch.full((M * Np + 32,), 0xEE, dtype=torch.uint8, device=DEV)
    ws = torch.empty(max(256, B.fpq_gemm_workspace_size(M, N, K, 0)), dtype=torch.uint8, device=DEV)
    sd = dev(np.array([sy], dtype=np.float32)) if sy_on_device else None
    B.fpq_gemm_codes_out(dev(xq), 0, fx, sx, None, packed, fw, sw_t, None if bias is None else dev(bias), fy,
                         0.0 if sy_on_device else sy, sd, buf[16:], M, N, K, acc, ws)
    torch.cuda.synchronize()
    h = buf.cpu().numpy()
    assert np.all(h[:16] == 0xEE) and np.all(h[16 + M * Np:] == 0xEE), "written outside the code matrix"
    return h[16:16 + M * Np].reshape(M, Np)


# generic kernel (small or N % 160 != 0), 128-row tile, 128-row tile with a ragged last tile, split K, 256-row tile
LINEAR = [(5, 48, 3), (77, 768, 320), (130, 128, 65), (200, 1280, 130), (8192, 320, 320), (8200, 320, 480), (300, 2880, 320),
          (512, 6400, 160), (24576, 2048, 320)]


@pytest.mark.parametrize("M,K,N", LINEAR)
@pytest.mark.parametrize("fw,fy,acc", [(E4M3, E4M3, 0), (E2M1, E4M3, 0), (E2M1, E3M4, 0), (E4M3, E5M2, 1), (E2M1, E4M3, 1)])
def test_linear_codes_out(M, K, N, fw, fy, acc):
    fx = E4M3
    x = synth.activations((M, K), 5000 + M)
    w = synth.weights((N, K), 5500 + N)
    h = synth.rounding_mask((N, K), 5750 + N) if fw is E2M1 else None
    bias = np.linspace(-1, 1, N).astype(np.float32)
    sx, xq, wq, sw = oracle_linear_inputs(x, w, h, fx, fw)
    Y, T = oracle.gemm(xq, fx, sx, wq, fw, sw, bias)
    sy = out_scale(Y, fy)
    packed, sw_t, _ = gpu_pack(w, fw, h, want_codes=False)
    got = gpu_linear_codes(xq, sx, fx, packed, fw, sw_t, bias, fy, sy, M, N, K, acc, sy_on_device=(M % 2 == 1))
    miss = check_codes(got, Y, T, fy, sy, REL_FP8_MFMA if acc else 1e-5, "linear codes out %s" % ((M, K, N, fw, fy, acc),))
    if not acc:
        assert miss < 0.002


@pytest.mark.parametrize("M,N", [(64, 48), (300, 160), (8192, 320), (8200, 320)])
@pytest.mark.parametrize("f", [E4M3, E3M4, E5M2])
def test_identity_layer_returns_its_input_codes(M, N, f):
    """Weights = identity (code of 1.0, scale 1), output format and scale = input format and scale: every sum has one
    non-zero term and is exact, so the codes that come out are the codes that went in (-0 aside: a sum of zeros of
    both signs is +0)."""
    rng = np.random.default_rng(M + N)
    xq = rng.integers(0, 256, size=(M, N), dtype=np.uint8)
    if f is E4M3:
        xq[(xq & 0x7F) == 0x7F] = 0x7E          # (4, 3, 7, 448): the all-ones magnitude is not a code of the format
    if f is E5M2:
        xq[(xq & 0x7C) == 0x7C] = 0x7B          # (5, 2, 15, 57344): nor is the top exponent
    xq[xq == (1 << (f[0] + f[1]))] = 0
    sx = 0.037
    w = np.eye(N, dtype=np.float32)
    packed, sw_t, _ = gpu_pack(w, f, None, scale_np=np.ones(N, dtype=np.float32), want_codes=False)
    got = gpu_linear_codes(xq, sx, f, packed, f, sw_t, None, f, sx, M, N, N, B.FPQ_ACC_FP32)
    assert np.array_equal(got[:, :N], xq)
    wq, sw = oracle.pack_weights(w, f, None, np.ones(N, dtype=np.float32))
    Y, _ = oracle.gemm(xq, f, sx, wq, f, sw)
    assert np.array_equal(oracle.requantize(Y, f, sx), xq)


@pytest.mark.parametrize("M,N", [(64, 48), (8192, 320), (8200, 480)])
@pytest.mark.parametrize("fy", [E4M3, E5M2, E3M4, synth.E2M5, (4, 3, 7, 240.0), (4, 3, 9, 112.0)])
@pytest.mark.parametrize("ratio", [0.37, 3.3, 150.0])
def test_epilogue_quantizer_bit_exact_on_single_term_sums(M, N, fy, ratio):
    """Identity weights: every output is one product x * sx, rounded to fp32 once on both sides, so the codes of the
    epilogue's quantizer (hardware conversion for E4M3 / E5M2, arithmetic encoder otherwise) must equal the oracle's
    bit for bit, whatever the output format and scale: clipped values, ties, subnormals, results that round to zero
    with either sign."""
    f = E4M3
    rng = np.random.default_rng(M + N)
    xq = rng.integers(0, 256, size=(M, N), dtype=np.uint8)
    xq[(xq & 0x7F) == 0x7F] = 0x7E
    xq[xq == 0x80] = 0
    sx = 0.0371
    sy = float(np.float32(sx * ratio * f[3] / fy[3]))
    w = np.eye(N, dtype=np.float32)
    packed, sw_t, _ = gpu_pack(w, f, None, scale_np=np.ones(N, dtype=np.float32), want_codes=False)
    got = gpu_linear_codes(xq, sx, f, packed, f, sw_t, None, fy, sy, M, N, N, B.FPQ_ACC_FP32)
    wq, sw = oracle.pack_weights(w, f, None, np.ones(N, dtype=np.float32))
    Y, _ = oracle.gemm(xq, f, sx, wq, f, sw)
    want = oracle.requantize(Y, fy, sy)
    assert np.array_equal(got[:, :N], want), int((got[:, :N] != want).sum())
    assert len(np.unique(want)) > 4


def check_codes_interval(got, O, tol, fy, sy, what):
    """got: uint8 [M, No]; O: exact result of the whole epilogue (double), tol: its error bound per element."""
    lo = oracle.quantize(np.nextafter((O - tol).astype(np.float32), np.float32(-np.inf)), fy, sy)
    hi = oracle.quantize(np.nextafter((O + tol).astype(np.float32), np.float32(np.inf)), fy, sy)
    vlo, vhi, vg = (oracle.dequantize(c, fy) for c in (lo, hi, got))
    bad = (vg < vlo) | (vg > vhi)
    assert not bad.any(), "%s: %d of %d codes outside the tolerance interval" % (what, int(bad.sum()), bad.size)
    same = lo == hi
    assert np.array_equal(got[same], lo[same]), what
    return float((got != oracle.requantize(O, fy, sy)).mean())


# generic kernel, 128-row tile (whole and ragged), split K, 256-row tile; N % 32 == 0 for the gated form
ACT_SHAPES = [(77, 768, 320), (130, 128, 64), (8192, 320, 320), (8200, 320, 640), (300, 2880, 320), (24576, 2048, 320)]


@pytest.mark.parametrize("M,K,N", ACT_SHAPES)
@pytest.mark.parametrize("fw,fy,acc", [(E4M3, E4M3, 0), (E2M1, E3M4, 0), (E2M1, E4M3, 1)])
@pytest.mark.parametrize("act", ["silu", "geglu"])
def test_linear_activation_then_codes(M, K, N, fw, fy, acc, act):
    fx = E4M3
    x = synth.activations((M, K), 7000 + M)
    w = synth.weights((N, K), 7500 + N) * 4.0          # results of order 1, where the activations bend
    h = synth.rounding_mask((N, K), 7750 + N) if fw is E2M1 else None
    bias = np.linspace(-1, 1, N).astype(np.float32)
    sx, xq, wq, sw = oracle_linear_inputs(x, w, h, fx, fw)
    Y, T = oracle.gemm(xq, fx, sx, wq, fw, sw, bias)
    t = (REL_FP8_MFMA if acc else 1e-5) * T + 1e-6
    if act == "silu":
        O = oracle.silu(Y)
        tol = 1.1 * t + 1e-6 * np.abs(O) + 1e-12        # |silu'| <= 1.1; fp32 evaluation of the activation
        flag, No = B.FPQ_ACT_SILU, N
    else:
        O = oracle.geglu(Y)
        Yb, tb = Y.reshape(M, N // 32, 2, 16), t.reshape(M, N // 32, 2, 16)
        a, g, ta, tg = Yb[:, :, 0, :], Yb[:, :, 1, :], tb[:, :, 0, :], tb[:, :, 1, :]
        G = oracle.gelu(g)
        dG = 1.13 * tg + 4e-7 * np.abs(g) + 1e-6 * np.abs(G) + 1e-12      # |gelu'| <= 1.13; the kernel's erf approximation
        tol = (np.abs(G) * ta + (np.abs(a) + ta) * dG + 1e-6 * np.abs(a * G)).reshape(M, N // 2)
        flag, No = B.FPQ_ACT_GEGLU, N // 2
    sy = out_scale(O, fy)
    packed, sw_t, _ = gpu_pack(w, fw, h, want_codes=False)
    Np = B.fpq_padded_channels(No)
    buf = torch.full((M * Np + 32,), 0xEE, dtype=torch.uint8, device=DEV)
    ws = torch.empty(max(256, B.fpq_gemm_workspace_size(M, N, K, 0)), dtype=torch.uint8, device=DEV)
    B.fpq_gemm_codes_out(dev(xq), 0, fx, sx, None, packed, fw, sw_t, dev(bias), fy, sy, None, buf[16:], M, N, K, acc | flag, ws)
    torch.cuda.synchronize()
    hb = buf.cpu().numpy()
    assert np.all(hb[:16] == 0xEE) and np.all(hb[16 + M * Np:] == 0xEE), "written outside the code matrix"
    got = hb[16:16 + M * Np].reshape(M, Np)
    assert np.all(got[:, No:] == 0)
    miss = check_codes_interval(got[:, :No], O, tol, fy, sy, "%s then codes %s" % (act, (M, K, N, fw, fy, acc)))
    if not acc:
        assert miss < 0.005


def test_gated_projection_given_in_the_plain_values_then_gates_layout():
    """A feed-forward projection as a model stores it, all value channels before all gate channels.  The caller
    reorders the weight rows (and the bias) once into blocks of 16 values + 16 gates, as the header of the gated
    form asks; the codes that come out are then, column for column, those of the block's own definition
    values * gelu(gates) evaluated by the oracle on the result of the layer with the weights as stored."""
    M, K, N = 300, 320, 640
    fx, fw, fy = E4M3, E2M1, E4M3
    x = synth.activations((M, K), 9001)
    w = synth.weights((N, K), 9501) * 4.0
    h = synth.rounding_mask((N, K), 9751)
    bias = np.linspace(-1, 1, N).astype(np.float32)
    sx, xq, wq, sw = oracle_linear_inputs(x, w, h, fx, fw)
    Y, T = oracle.gemm(xq, fx, sx, wq, fw, sw, bias)                  # plain layout
    O = oracle.geglu_plain(Y)
    t = 1e-5 * T + 1e-6
    half = N // 2
    a, g, ta, tg = Y[:, :half], Y[:, half:], t[:, :half], t[:, half:]
    G = oracle.gelu(g)
    dG = 1.13 * tg + 4e-7 * np.abs(g) + 1e-6 * np.abs(G) + 1e-12
    tol = np.abs(G) * ta + (np.abs(a) + ta) * dG + 1e-6 * np.abs(a * G)
    sy = out_scale(O, fy)
    order = oracle.geglu_interleaved_rows(N)                           # the caller's one-time reordering
    packed, sw_t, _ = gpu_pack(w[order], fw, h[order], want_codes=False)
    assert np.array_equal(sw_t.cpu().numpy(), sw[order])               # per-channel scales move with their rows
    yq = torch.full((M, half), 0xEE, dtype=torch.uint8, device=DEV)
    ws = torch.empty(max(256, B.fpq_gemm_workspace_size(M, N, K, 0)), dtype=torch.uint8, device=DEV)
    B.fpq_gemm_codes_out(dev(xq), 0, fx, sx, None, packed, fw, sw_t, dev(bias[order]), fy, sy, None, yq, M, N, K,
                         B.FPQ_ACC_FP32 | B.FPQ_ACT_GEGLU, ws)
    torch.cuda.synchronize()
    miss = check_codes_interval(yq.cpu().numpy(), O, tol, fy, sy, "plain-layout gated projection")
    assert miss < 0.005


def test_feed_forward_projection_at_full_size_sampled_rows():
    """The transformer-block projection of configuration 3 (16384 x 320 -> 2560) as the U-Net runs it: gated GELU, then
    codes for the output layer.  All of it runs on the GPU in the bench's launch configuration; the oracle computes
    tile-corner and random rows one by one."""
    M, K, N = 16384, 320, 2560
    fx, fw, fy = E4M3, E2M1, E4M3
    x = synth.activations((M, K), 3001)
    w = synth.weights((N, K), 3501) * 4.0
    h = synth.rounding_mask((N, K), 3751)
    bias = np.linspace(-1, 1, N).astype(np.float32)
    sx, xq, wq, sw = oracle_linear_inputs(x, w, h, fx, fw)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 127, 128, 255, 256, M - 129, M - 128, M - 1], rng.integers(0, M, 120)]))
    Y, T = oracle.gemm(xq, fx, sx, wq, fw, sw, bias, rows=rows)
    t = 1e-5 * T + 1e-6
    O = oracle.geglu(Y)
    R = len(rows)
    Yb, tb = Y.reshape(R, N // 32, 2, 16), t.reshape(R, N // 32, 2, 16)
    a, g, ta, tg = Yb[:, :, 0, :], Yb[:, :, 1, :], tb[:, :, 0, :], tb[:, :, 1, :]
    G = oracle.gelu(g)
    dG = 1.13 * tg + 4e-7 * np.abs(g) + 1e-6 * np.abs(G) + 1e-12
    tol = (np.abs(G) * ta + (np.abs(a) + ta) * dG + 1e-6 * np.abs(a * G)).reshape(R, N // 2)
    sy = out_scale(O, fy)
    packed, sw_t, _ = gpu_pack(w, fw, h, want_codes=False)
    yq = torch.full((M, N // 2), 0xEE, dtype=torch.uint8, device=DEV)
    ws = torch.empty(max(256, B.fpq_gemm_workspace_size(M, N, K, 0)), dtype=torch.uint8, device=DEV)
    B.fpq_gemm_codes_out(dev(xq), 0, fx, sx, None, packed, fw, sw_t, dev(bias), fy, sy, None, yq, M, N, K,
                         B.FPQ_ACC_FP32 | B.FPQ_ACT_GEGLU, ws)
    torch.cuda.synchronize()
    got = yq.cpu().numpy()
    miss = check_codes_interval(got[rows], O, tol, fy, sy, "config-3 projection, gated, codes out")
    assert miss < 0.005
    # and the codes feed the output layer (1280 -> 320) as they stand
    N2 = 320
    w2 = synth.weights((N2, N // 2), 3502)
    wq2, sw2 = oracle.pack_weights(w2, E4M3, None)
    packed2, sw2_t, _ = gpu_pack(w2, E4M3, None, want_codes=False)
    y2 = torch.full((M, N2), float("nan"), device=DEV)
    ws2 = torch.empty(max(256, B.fpq_gemm_workspace_size(M, N2, N // 2, 0)), dtype=torch.uint8, device=DEV)
    B.fpq_gemm(yq, 0, fy, sy, None, packed2, E4M3, sw2_t, None, y2, M, N2, N // 2, B.FPQ_ACC_FP32, ws2)
    torch.cuda.synchronize()
    Y2, T2 = oracle.gemm(got, fy, sy, wq2, E4M3, sw2, None, rows=rows)
    assert np.all(np.abs(y2.cpu().numpy()[rows] - Y2) <= 1e-5 * T2 + 1e-6)


@pytest.mark.parametrize("case", [(2, 32, 5, 5, 64, 1, 1, 0), (1, 48, 12, 10, 130, 3, 1, 0), (2, 64, 65, 63, 160, 3, 2, 1),
                                  (1, 640, 16, 16, 160, 3, 1, 1)])
def test_conv_silu_then_codes(case):
    Bn, Cin, H, W, Cout, k, stride, pad = case
    fx = fw = fy = E4M3
    x = synth.activations((Bn, Cin, H, W), 8000 + Cin)
    w = synth.weights((Cout, Cin, k, k), 8500 + Cout) * 4.0
    bias = np.linspace(-0.5, 0.5, Cout).astype(np.float32)
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, None)
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    M = Bn * Ho * Wo
    Y, T = oracle.conv2d(xq, fx, sx, wq, fw, sw, bias, stride=stride, pad=pad)
    Y = Y.transpose(0, 2, 3, 1).reshape(M, Cout)
    T = T.transpose(0, 2, 3, 1).reshape(M, Cout)
    O = oracle.silu(Y)
    tol = 1.1 * (1e-5 * T + 1e-6) + 1e-6 * np.abs(O) + 1e-12
    sy = out_scale(O, fy)
    packed, sw_t, _ = gpu_pack(w, fw, None, want_codes=False)
    Cp, Np = B.fpq_padded_channels(Cin), B.fpq_padded_channels(Cout)
    codes_in = torch.empty(Bn * H * W * Cp, dtype=torch.uint8, device=DEV)
    B.fpq_quantize_nhwc(dev(x), fx, sx, None, codes_in)
    buf = torch.full((M * Np + 32,), 0xEE, dtype=torch.uint8, device=DEV)
    ws = torch.empty(max(256, B.fpq_conv2d_workspace_size(Bn, Cin, H, W, Cout, k, k, stride, pad, 0)), dtype=torch.uint8,
                     device=DEV)
    B.fpq_conv2d_codes_out(codes_in, 0, fx, sx, None, packed, fw, sw_t, dev(bias), fy, sy, None, buf[16:], Bn, Cin, H, W,
                           Cout, k, k, stride, pad, B.FPQ_ACC_FP32 | B.FPQ_ACT_SILU, ws)
    torch.cuda.synchronize()
    hb = buf.cpu().numpy()
    assert np.all(hb[:16] == 0xEE) and np.all(hb[16 + M * Np:] == 0xEE)
    got = hb[16:16 + M * Np].reshape(M, Np)
    assert np.all(got[:, Cout:] == 0)
    check_codes_interval(got[:, :Cout], O, tol, fy, sy, "conv silu then codes %s" % (case,))


CONVS = [  # B, Cin, H, W, Cout, k, stride, pad: generic kernels, large tile, large tile with split K
    (2, 4, 9, 7, 5, 3, 1, 1), (1, 20, 6, 6, 33, 3, 2, 1), (2, 32, 5, 5, 64, 1, 1, 0), (1, 48, 12, 10, 130, 3, 1, 0),
    (2, 320, 64, 64, 320, 3, 1, 1), (2, 64, 65, 63, 160, 3, 2, 1), (1, 640, 16, 16, 160, 3, 1, 1), (8, 320, 32, 32, 320, 1, 1, 0),
]


@pytest.mark.parametrize("case", CONVS)
@pytest.mark.parametrize("fw,fy,acc", [(E4M3, E4M3, 0), (E2M1, E4M3, 0), (E2M1, E3M4, 1)])
def test_conv_codes_out_feed_the_next_layer(case, fw, fy, acc):
    Bn, Cin, H, W, Cout, k, stride, pad = case
    fx = E4M3
    x = synth.activations((Bn, Cin, H, W), 6000 + Cin)
    w = synth.weights((Cout, Cin, k, k), 6500 + Cout)
    h = synth.rounding_mask(w.shape, 6750 + Cout) if fw is E2M1 else None
    bias = np.linspace(-0.5, 0.5, Cout).astype(np.float32)
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    M = Bn * Ho * Wo
    pix = None
    if M * Cout * Cin * k * k > 3e9:                      # the oracle computes a sample of the pixels one by one
        rng = np.random.default_rng(Cin)
        pix = np.unique(np.concatenate([np.arange(0, M, 127), [M - 1, 255, 256], rng.integers(0, M, 400)]))
    Y, T = oracle.conv2d(xq, fx, sx, wq, fw, sw, bias, stride=stride, pad=pad, pix=pix)
    if pix is None:
        Y = Y.transpose(0, 2, 3, 1).reshape(M, Cout)       # channels-last rows, as the codes are laid out
        T = T.transpose(0, 2, 3, 1).reshape(M, Cout)
    sy = out_scale(Y, fy)
    packed, sw_t, _ = gpu_pack(w, fw, h, want_codes=False)
    Cp, Np = B.fpq_padded_channels(Cin), B.fpq_padded_channels(Cout)
    codes_in = torch.empty(Bn * H * W * Cp, dtype=torch.uint8, device=DEV)
    B.fpq_quantize_nhwc(dev(x), fx, sx, None, codes_in)
    buf = torch.full((M * Np + 32,), 0xEE, dtype=torch.uint8, device=DEV)
    ws = torch.empty(max(256, B.fpq_conv2d_workspace_size(Bn, Cin, H, W, Cout, k, k, stride, pad, 0)), dtype=torch.uint8,
                     device=DEV)
    B.fpq_conv2d_codes_out(codes_in, 0, fx, sx, None, packed, fw, sw_t, dev(bias), fy, sy, None, buf[16:], Bn, Cin, H, W,
                           Cout, k, k, stride, pad, acc, ws)
    torch.cuda.synchronize()
    hb = buf.cpu().numpy()
    assert np.all(hb[:16] == 0xEE) and np.all(hb[16 + M * Np:] == 0xEE)
    got = hb[16:16 + M * Np].reshape(M, Np)
    rel = REL_FP8_MFMA if acc else 1e-5
    check_codes(got if pix is None else got[pix], Y, T, fy, sy, rel, "conv codes out %s" % ((case, fw, fy, acc),))

    # the code buffer is the next convolution's channels-last input as it stands: a 1x1 layer on it must equal the
    # oracle's layer on the same codes (whatever they are)
    if fy is E4M3 and Cout <= 320:
        N2 = 48
        w2 = synth.weights((N2, Cout, 1, 1), 6900 + Cout)
        wq2, sw2 = oracle.pack_weights(w2, E4M3, None)
        packed2, sw2_t, _ = gpu_pack(w2, E4M3, None, want_codes=False)
        y2 = torch.full((Bn, N2, Ho, Wo), float("nan"), dtype=torch.float32, device=DEV)
        ws2 = torch.empty(max(256, B.fpq_conv2d_workspace_size(Bn, Cout, Ho, Wo, N2, 1, 1, 1, 0, 0)), dtype=torch.uint8,
                          device=DEV)
        B.fpq_conv2d(buf[16:], 0, fy, sy, None, packed2, E4M3, sw2_t, None, y2, Bn, Cout, Ho, Wo, N2, 1, 1, 1, 0,
                     B.FPQ_ACC_FP32, ws2)
        torch.cuda.synchronize()
        xq2 = got[:, :Cout].reshape(Bn, Ho, Wo, Cout).transpose(0, 3, 1, 2)
        rows = np.unique(np.concatenate([np.arange(0, M, max(1, M // 64)), [M - 1]]))
        Y2, T2 = oracle.conv2d(np.ascontiguousarray(xq2), fy, sy, wq2, E4M3, sw2, None, stride=1, pad=0, pix=rows)
        y2h = y2.cpu().numpy().transpose(0, 2, 3, 1).reshape(M, N2)[rows]
        err = np.abs(y2h - Y2)
        assert np.all(err <= 1e-5 * T2 + 1e-6)


def test_codes_out_argument_checks():
    p = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    f = B.fmt(E4M3)
    L = B.lib()
    import ctypes as C
    P = C.c_void_p(p.data_ptr())
    assert L.fpq_gemm_codes_out(P, 0, f, 1.0, None, P, f, P, None, B.fmt(E2M1), 1.0, None, P, 8, 8, 32, 0, None, 0, None) == -8
    assert L.fpq_gemm_codes_out(P, 0, f, 1.0, None, P, f, P, None, f, 0.0, None, P, 8, 8, 32, 0, None, 0, None) == -3
    assert L.fpq_gemm_codes_out(P, 0, f, 1.0, None, P, f, P, None, f, 1.0, None, None, 8, 8, 32, 0, None, 0, None) == -1
    assert L.fpq_gemm_codes_out(P, 0, f, 1.0, None, P, f, P, None, f, 1.0, None, P, 8, 8, 32, B.FPQ_OUT_ACCUMULATE, None, 0,
                                None) == -8
    assert L.fpq_gemm_codes_out(P, 0, f, 1.0, None, P, f, P, None, f, 1.0, None, C.c_void_p(p.data_ptr() + 4), 8, 8, 32, 0,
                                None, 0, None) == -5
    # activations: only with codes out, one at a time, the gated one for linear layers with N % 32 == 0
    y = torch.zeros(64, device=DEV)
    Y = C.c_void_p(y.data_ptr())
    assert L.fpq_gemm(P, 0, f, 1.0, None, P, f, P, None, Y, 8, 8, 32, B.FPQ_ACT_SILU, None, 0, None) == -8
    assert L.fpq_gemm_codes_out(P, 0, f, 1.0, None, P, f, P, None, f, 1.0, None, P, 8, 8, 32, B.FPQ_ACT_GEGLU, None, 0, None) == -8
    assert L.fpq_gemm_codes_out(P, 0, f, 1.0, None, P, f, P, None, f, 1.0, None, P, 8, 32, 32,
                                B.FPQ_ACT_GEGLU | B.FPQ_ACT_SILU, None, 0, None) == -8
    assert L.fpq_conv2d_codes_out(P, 0, f, 1.0, None, P, f, P, None, f, 1.0, None, P, 1, 16, 4, 4, 32, 1, 1, 1, 0,
                                  B.FPQ_ACT_GEGLU, None, 0, None) == -8
