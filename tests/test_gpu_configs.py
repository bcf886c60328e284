"""GPU parity at the full sizes of the five workload configurations, through the same entry points and
launch configuration that bench.py times (absmax on the device -> device-resident scale -> fused
quantize + layer call).  Outputs are compared in full where the oracle finishes in seconds and on a
sample of output rows / pixels (tile corners, borders and random positions) otherwise."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, check_close, dev

pytestmark = pytest.mark.gpu
REL_FP8_MFMA = 7 * 2.0 ** -13


def sample_positions(M, n_random, seed, tile=128):
    """First / last row of every tile plus random rows."""
    edges = np.unique(np.concatenate([np.arange(0, M, tile), np.minimum(np.arange(0, M, tile) + tile - 1, M - 1)]))
    rng = np.random.default_rng(seed)
    rnd = rng.integers(0, M, n_random)
    return np.unique(np.concatenate([edges, rnd, [0, M - 1]]))


def run_layer_gpu(L, x_t, w_t, h_t, fx, fw, acc, bias_t=None):
    """The bench's call sequence for one layer; returns (y, scale, activation codes buffer, weight codes)."""
    kk = L.k if L.kind == "conv" else 1
    wshape = (L.Cout, L.Cin, kk, kk)
    packed = torch.empty(B.fpq_packed_size(L.N, L.Cin, kk, kk, fw), dtype=torch.uint8, device=DEV)
    sw = torch.empty(L.N, dtype=torch.float32, device=DEV)
    wcodes = torch.empty(L.N * L.K, dtype=torch.uint8, device=DEV)
    B.fpq_pack_weights(w_t.reshape(wshape), fw, None, h_t, packed, sw, wcodes)
    y = torch.full((L.M * L.N,), float("nan"), dtype=torch.float32, device=DEV)
    # dynamic-scale mode (what bench.py calls): absmax, scale, quantize and the layer in one call
    if L.kind == "conv":
        ws = torch.empty(B.fpq_conv2d_workspace_size(L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad, 2),
                         dtype=torch.uint8, device=DEV)
        B.fpq_conv2d(x_t, B.FPQ_X_FP32_DYNAMIC, fx, 0.0, None, packed, fw, sw, bias_t, y, L.B, L.Cin, L.H, L.W, L.Cout,
                     L.k, L.k, L.stride, L.pad, acc, ws)
    else:
        ws = torch.empty(B.fpq_gemm_workspace_size(L.M, L.N, L.K, 2), dtype=torch.uint8, device=DEV)
        B.fpq_gemm(x_t, B.FPQ_X_FP32_DYNAMIC, fx, 0.0, None, packed, fw, sw, bias_t, y, L.M, L.N, L.K, acc, ws)
    torch.cuda.synchronize()
    # the workspace ends with 1024 partial maxima and a 256-byte slot holding [scale, absmax]
    pub = ws[-256:-248].view(torch.float32)
    sc = torch.stack([pub[1], pub[0]])
    torch.cuda.synchronize()
    return y, sc.cpu().numpy(), ws, wcodes, sw


def check_layer(L, x, w, h, fx, fw, accs, n_random=64, seed=0, full=False):
    """x, w, h: host arrays.  Runs the GPU path and the oracle; compares scale, codes and outputs."""
    x_t, w_t = dev(x), dev(w)
    h_t = None if h is None else dev(h)
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    bias = np.linspace(-0.3, 0.3, L.N).astype(np.float32)
    pos = None if full else sample_positions(L.M, n_random, seed)
    if L.kind == "conv":
        Y, T = oracle.conv2d(xq, fx, sx, wq.reshape(L.Cout, L.Cin, L.k, L.k), fw, sw, bias, stride=L.stride, pad=L.pad,
                             pix=pos)
    else:
        Y, T = oracle.gemm(xq, fx, sx, wq.reshape(L.N, L.K), fw, sw, bias, rows=pos)
    worst = {}
    for acc in accs:
        y, sc, ws, wcodes, sw_t = run_layer_gpu(L, x_t, w_t, h_t, fx, fw, acc, dev(bias))
        assert sc[0] == np.float32(oracle.absmax(x)) and sc[1] == np.float32(sx)
        assert np.array_equal(wcodes.cpu().numpy(), wq.reshape(-1)), "weight codes"
        assert np.array_equal(sw_t.cpu().numpy(), sw)
        # activation codes as the layer consumed them
        if L.kind == "conv":
            Cp = B.fpq_padded_channels(L.Cin)
            got = ws.cpu().numpy()[:L.B * L.H * L.W * Cp].reshape(L.B, L.H, L.W, Cp)
            assert np.array_equal(got[..., :L.Cin], xq.transpose(0, 2, 3, 1)), "activation codes"
            yv = y.cpu().numpy().reshape(L.B, L.Cout, -1)
            if full:
                got_y = yv.reshape(Y.shape)
            else:
                hw = yv.shape[2]
                got_y = yv[pos // hw, :, pos % hw]
        else:
            # small linear layers quantize inside the layer kernel's loader and leave no codes behind: check
            # the quantizer on its own with the scale the call published
            qc = torch.empty(L.M * L.K, dtype=torch.uint8, device=DEV)
            B.fpq_quantize(x_t, fx, 0.0, ws[-256:-252].view(torch.float32), qc)
            torch.cuda.synchronize()
            assert np.array_equal(qc.cpu().numpy().reshape(L.M, L.K), xq), "activation codes"
            yv = y.cpu().numpy().reshape(L.M, L.N)
            got_y = yv if full else yv[pos]
        assert not np.isnan(y.cpu().numpy()).any(), "unwritten outputs"
        worst[acc] = check_close(got_y, Y, T, rel=REL_FP8_MFMA if acc == B.FPQ_ACC_FP8_MFMA else 1e-5,
                                 what="%s acc %d" % (L.name, acc))
    return worst


def host_inputs(L, cfg, li=0):
    sx_seed, sw_seed, sh_seed = synth.seeds(cfg, li)
    kk = L.k if L.kind == "conv" else 1
    x = synth.activations((L.B, L.Cin, L.H, L.W) if L.kind == "conv" else (L.M, L.K), sx_seed)
    w = synth.weights((L.Cout, L.Cin, kk, kk), sw_seed)
    h = synth.rounding_mask(w.shape, sh_seed)
    return x, w, h


def test_config1_linear_w8a8_full():
    L = synth.config_layers(1)[0]
    x, w, h = host_inputs(L, 1)
    check_layer(L, x, w, h, synth.E4M3, synth.E4M3, (B.FPQ_ACC_FP32, B.FPQ_ACC_FP8_MFMA), full=True)
    check_layer(L, x, w, h, synth.E4M3, synth.E2M1, (B.FPQ_ACC_FP32,), full=True)


def test_config2_conv_w8a8_full():
    L = synth.config_layers(2)[0]
    x, w, h = host_inputs(L, 2)
    check_layer(L, x, w, h, synth.E4M3, synth.E4M3, (B.FPQ_ACC_FP32, B.FPQ_ACC_FP8_MFMA), full=True)


@pytest.mark.parametrize("li", range(5))
def test_config3_projections(li):
    L = synth.config_layers(3)[li]
    x, w, h = host_inputs(L, 3, li)
    check_layer(L, x, w, h, synth.E4M3, synth.E4M3, (B.FPQ_ACC_FP32, B.FPQ_ACC_FP8_MFMA), n_random=256, seed=li,
                full=(L.M < 1000))


def test_config4_conv_w4a8_and_non_native_sweep():
    L = synth.config_layers(4)[0]
    x, w, h = host_inputs(L, 4)
    check_layer(L, x, w, h, synth.E4M3, synth.E2M1, (B.FPQ_ACC_FP32, B.FPQ_ACC_FP8_MFMA), n_random=400, seed=4)
    check_layer(L, x, w, h, synth.E3M4, synth.E3M0, (B.FPQ_ACC_FP32,), n_random=200, seed=5)


# ---- configuration 5: one representative of every distinct layer shape of the 250-layer set

def layer_class(L):
    return (L.kind, L.k if L.kind == "conv" else 1, L.stride if L.kind == "conv" else 1, L.M, L.K, L.N)


def layer_plan(L):
    """(kernel, K slices) the library states for this layer's shape."""
    if L.kind == "conv":
        return B.fpq_conv2d_plan(L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad)
    return B.fpq_gemm_plan(L.M, L.N, L.K)


def cfg5_classes():
    """[(index of the first layer of the class in the layer list, layer)] in order of first appearance."""
    seen, out = set(), []
    for li, L in enumerate(synth.unet_layers()):
        c = layer_class(L)
        if c not in seen:
            seen.add(c)
            out.append((li, L))
    return out


CFG5_CLASSES = cfg5_classes()
PLANS_RUN = set()   # (layer kind, kernel, K slices) of the class tests that have run in this process


def sample_positions_large(M, seed):
    """Rows for a layer too large to compare on every tile: first and last row of the first, the last and 24 random
    128-row tiles (which are also the corners of the 256-row tiles they fall in), plus 32 random rows."""
    if M <= 4096:
        return sample_positions(M, 32, seed)
    rng = np.random.default_rng(seed)
    nt = (M + 127) // 128
    tiles = np.unique(np.concatenate([[0, nt - 1], rng.integers(0, nt, 24)]))
    rows = np.concatenate([tiles * 128, np.minimum(tiles * 128 + 127, M - 1), rng.integers(0, M, 32), [0, M - 1]])
    return np.unique(rows)


def check_layer_rows(L, x, w, h, fx, fw, acc, pos, what):
    """As check_layer, on the given output rows / pixels, one accumulate mode, without re-checking the operand codes."""
    x_t, w_t = dev(x), dev(w)
    h_t = None if h is None else dev(h)
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    bias = np.linspace(-0.3, 0.3, L.N).astype(np.float32)
    if L.kind == "conv":
        Y, T = oracle.conv2d(xq, fx, sx, wq.reshape(L.Cout, L.Cin, L.k, L.k), fw, sw, bias, stride=L.stride, pad=L.pad,
                             pix=pos)
    else:
        Y, T = oracle.gemm(xq, fx, sx, wq.reshape(L.N, L.K), fw, sw, bias, rows=pos)
    y, sc, ws, wcodes, sw_t = run_layer_gpu(L, x_t, w_t, h_t, fx, fw, acc, dev(bias))
    assert sc[0] == np.float32(oracle.absmax(x)) and sc[1] == np.float32(sx), what
    assert np.array_equal(wcodes.cpu().numpy(), wq.reshape(-1)), "weight codes " + what
    assert np.array_equal(sw_t.cpu().numpy(), sw), what
    yh = y.cpu().numpy()
    assert not np.isnan(yh).any(), "unwritten outputs " + what
    if L.kind == "conv":
        yv = yh.reshape(L.B, L.Cout, -1)
        hw = yv.shape[2]
        got_y = yv[pos // hw, :, pos % hw]
    else:
        got_y = yh.reshape(L.M, L.N)[pos]
    return check_close(got_y, Y, T, rel=1e-5, what=what)


@pytest.mark.parametrize("li,L", CFG5_CLASSES, ids=["%03d_%s" % (li, L.name) for li, L in CFG5_CLASSES])
def test_config5_every_shape_class(li, L):
    """Every distinct (kind, kernel size, stride, M, K, N) of the U-Net layer set at batch 8, with the inputs drawn on
    the device as bench.py draws them, through the bench's dynamic-scale call in the fp32-accumulate mode: W8A8
    (round-to-nearest E4M3 weights) and W4A8 (E2M1 weights with a rounding mask), on tile-corner and random rows the
    oracle computes one by one.  The launch configuration is the one the benchmark times for this class."""
    sx_seed, sw_seed, sh_seed = synth.seeds(5, li)
    kk = L.k if L.kind == "conv" else 1
    x_t = synth.activations_torch((L.B, L.Cin, L.H, L.W) if L.kind == "conv" else (L.M, L.K), sx_seed, DEV)
    w_t = synth.weights_torch((L.Cout, L.Cin, kk, kk), sw_seed, DEV)
    h_t = synth.rounding_mask_torch((L.Cout, L.Cin, kk, kk), sh_seed, DEV)
    x, w, h = x_t.cpu().numpy(), w_t.cpu().numpy(), h_t.cpu().numpy()
    del x_t, w_t, h_t
    pos = sample_positions_large(L.M, li)
    kernel, slices = layer_plan(L)
    # the slice count is visible from outside: the workspace of the codes form holds exactly the partial sums
    if L.kind == "conv":
        part = B.fpq_conv2d_workspace_size(L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad, 0)
    else:
        part = B.fpq_gemm_workspace_size(L.M, L.N, L.K, 0)
    want = slices * L.M * L.N * 4 if slices > 1 else 0
    assert part == (want + 255) // 256 * 256
    check_layer_rows(L, x, w, None, synth.E4M3, synth.E4M3, B.FPQ_ACC_FP32, pos, "%s W8A8" % L.name)
    check_layer_rows(L, x, w, h, synth.E4M3, synth.E2M1, B.FPQ_ACC_FP32, pos, "%s W4A8" % L.name)
    PLANS_RUN.add((L.kind, kernel, slices))


def test_config5_classes_cover_every_plan_of_the_layer_set():
    """The launch configurations (layer kind, kernel, K slices) of all 250 layers are exactly those of the class
    representatives above; and, when those tests ran in this process, exactly those that were compared."""
    layers = synth.unet_layers()
    assert len(layers) == 250 and len(CFG5_CLASSES) == len({layer_class(L) for L in layers})
    all_plans = {(L.kind,) + tuple(layer_plan(L)) for L in layers}
    class_plans = {(L.kind,) + tuple(layer_plan(L)) for _, L in CFG5_CLASSES}
    assert all_plans == class_plans
    assert any(k == B.FPQ_KERNEL_256x160 and s > 1 for _, k, s in all_plans), "the sliced 256-row plan is part of the set"
    if len(PLANS_RUN) >= len(class_plans):
        assert PLANS_RUN == all_plans
