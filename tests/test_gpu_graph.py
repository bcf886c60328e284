"""The layer entry points inside a captured HIP graph: every replay, with fresh inputs copied into the captured buffers
and eager work between the replays, must give what the eager call gives (bit for bit: same kernels, same order)."""
import numpy as np
import pytest
import torch

from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, dev, gpu_pack

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", ["conv_dynamic_splitk", "linear_dynamic", "linear_dynamic_8_rows", "linear_codes_out_geglu"])
def test_graph_replays_equal_eager(case):
    fx, fw = synth.E4M3, synth.E2M1
    if case == "conv_dynamic_splitk":
        shape, wshape = (1, 640, 16, 16), (160, 640, 3, 3)            # deep K, few tiles: K slices + reduction kernel
    elif case == "linear_dynamic_8_rows":
        shape, wshape = (8, 1280), (1280, 1280)                       # the one-launch form of the layers with <= 16 rows
    else:
        shape, wshape = (4096, 320), (640, 320)
    w = synth.weights(wshape, 31)
    packed, sw_t, _ = gpu_pack(w, fw, synth.rounding_mask(wshape, 32), want_codes=False)
    xs = [dev(synth.activations(shape, 40 + i)) for i in range(4)]
    x = torch.empty_like(xs[0])
    if case == "conv_dynamic_splitk":
        Bn, Cin, H, W = shape
        Cout = wshape[0]
        y = torch.empty((Bn, Cout, H, W), device=DEV)
        ws = torch.empty(B.fpq_conv2d_workspace_size(Bn, Cin, H, W, Cout, 3, 3, 1, 1, 2), dtype=torch.uint8, device=DEV)
        def call():
            B.fpq_conv2d(x, B.FPQ_X_FP32_DYNAMIC, fx, 0.0, None, packed, fw, sw_t, None, y, Bn, Cin, H, W, Cout, 3, 3, 1, 1,
                         B.FPQ_ACC_FP32, ws)
    elif case in ("linear_dynamic", "linear_dynamic_8_rows"):
        M, K = shape
        N = wshape[0]
        y = torch.empty((M, N), device=DEV)
        ws = torch.empty(B.fpq_gemm_workspace_size(M, N, K, 2), dtype=torch.uint8, device=DEV)
        def call():
            B.fpq_gemm(x, B.FPQ_X_FP32_DYNAMIC, fx, 0.0, None, packed, fw, sw_t, None, y, M, N, K, B.FPQ_ACC_FP32, ws)
    else:
        M, K = shape
        N = wshape[0]
        y = torch.empty((M, N // 2), dtype=torch.uint8, device=DEV)
        ws = torch.empty(B.fpq_gemm_workspace_size(M, N, K, 1), dtype=torch.uint8, device=DEV)
        def call():
            B.fpq_gemm_codes_out(x, B.FPQ_X_FP32, fx, 0.02, None, packed, fw, sw_t, None, fx, 0.01, None, y, M, N, K,
                                 B.FPQ_ACC_FP32 | B.FPQ_ACT_GEGLU, ws)
    # eager results for the four inputs
    want = []
    for xi in xs:
        x.copy_(xi)
        call()
        torch.cuda.synchronize()
        want.append(y.clone())
    assert not torch.equal(want[0], want[1])
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        x.copy_(xs[0])
        call()                                   # warm-up on the capture stream
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            call()
    torch.cuda.synchronize()
    for rep in range(8):
        i = (rep * 3 + 1) % 4
        x.copy_(xs[i])
        y.zero_()
        scratch = torch.randn(1 << 16, device=DEV).sum()      # unrelated eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want[i]), "replay %d differs from the eager result" % rep
        assert torch.isfinite(scratch)
