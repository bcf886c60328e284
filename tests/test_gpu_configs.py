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


CFG5_PICKS = ["time.fc1", "conv_in", "down0.res0.conv1", "down0.attn0.attn2.k", "down0.downsample", "down1.res0.skip",
              "down2.attn0.ff.geglu", "mid.res0.conv1", "up3.res0.conv1", "up2.res2.skip", "up0.res0.conv1",
              "up0.attn2.ff.out", "conv_out"]


@pytest.mark.parametrize("name", CFG5_PICKS)
def test_config5_sampled_layers(name):
    """Layers of the full U-Net set at batch 8, inputs drawn on the device as bench.py draws them."""
    layers = synth.unet_layers()
    li = [l.name for l in layers].index(name)
    L = layers[li]
    sx_seed, sw_seed, sh_seed = synth.seeds(5, li)
    kk = L.k if L.kind == "conv" else 1
    x_t = synth.activations_torch((L.B, L.Cin, L.H, L.W) if L.kind == "conv" else (L.M, L.K), sx_seed, DEV)
    w_t = synth.weights_torch((L.Cout, L.Cin, kk, kk), sw_seed, DEV)
    h_t = synth.rounding_mask_torch((L.Cout, L.Cin, kk, kk), sh_seed, DEV)
    x, w, h = x_t.cpu().numpy(), w_t.cpu().numpy(), h_t.cpu().numpy()
    big = synth.flops(L) > 2e10
    check_layer(L, x, w, None, synth.E4M3, synth.E4M3, (B.FPQ_ACC_FP32,), n_random=24 if big else 64, seed=li,
                full=(synth.flops(L) < 2e9))
    check_layer(L, x, w, h, synth.E4M3, synth.E2M1, (B.FPQ_ACC_FP32, B.FPQ_ACC_FP8_MFMA), n_random=24 if big else 64,
                seed=li + 1, full=(synth.flops(L) < 2e9))
