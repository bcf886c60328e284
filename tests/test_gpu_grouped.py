"""fpq_gemm_grouped: a group of independent linear layers in one call, against the oracle problem by problem, and
against fpq_gemm on the same problem (bit for bit where fpq_gemm itself uses the register-staged kernel)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, check_close, dev, gpu_pack

pytestmark = pytest.mark.gpu
E4M3, E2M1, E3M4, E3M0 = synth.E4M3, synth.E2M1, synth.E3M4, synth.E3M0


def make_problem(M, K, N, fx, fw, seed, with_bias):
    x = synth.activations((M, K), seed)
    w = synth.weights((N, K), seed + 1)
    h = synth.rounding_mask((N, K), seed + 2) if 1 + fw[0] + fw[1] <= 4 else None
    bias = np.linspace(-0.3, 0.3, N).astype(np.float32) if with_bias else None
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    Y, T = oracle.gemm(xq, fx, sx, wq, fw, sw, bias)
    packed, sw_t, _ = gpu_pack(w, fw, h, want_codes=False)
    return dict(M=M, K=K, N=N, x=x, xq=xq, sx=sx, Y=Y, T=T, packed=packed, sw_t=sw_t, x_t=dev(x),
                bias_t=None if bias is None else dev(bias),
                y=torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV))


def run_group_dynamic(ps, fx, fw, acc=B.FPQ_ACC_FP32):
    arr = B.gemm_problems([(p["x_t"], None, p["packed"], p["sw_t"], p["bias_t"], p["y"], p["M"], p["N"], p["K"]) for p in ps])
    need = B.fpq_gemm_grouped_workspace_size(arr, B.FPQ_X_FP32_DYNAMIC)
    assert need == sum((p["M"] * p["K"] + 255) // 256 * 256 + 256 for p in ps)
    ws = torch.full((need,), 0xEE, dtype=torch.uint8, device=DEV)
    B.fpq_gemm_grouped(arr, B.FPQ_X_FP32_DYNAMIC, fx, fw, acc, ws)
    torch.cuda.synchronize()
    return ws.cpu().numpy()


def check_group_dynamic(ps, fx, fw, ws, rel=1e-5):
    codes_at = 0
    slot_at = sum((p["M"] * p["K"] + 255) // 256 * 256 for p in ps)
    for i, p in enumerate(ps):
        n = p["M"] * p["K"]
        assert np.array_equal(ws[codes_at:codes_at + n].reshape(p["M"], p["K"]), p["xq"]), "codes of problem %d" % i
        pub = ws[slot_at + 128:slot_at + 136].view(np.float32)
        assert pub[0] == np.float32(p["sx"]) and pub[1] == np.float32(oracle.absmax(p["x"])), "scale of problem %d" % i
        yh = p["y"].cpu().numpy()
        assert not np.isnan(yh).any(), "unwritten outputs in problem %d" % i
        check_close(yh, p["Y"], p["T"], rel=rel, what="grouped problem %d %s" % (i, (p["M"], p["K"], p["N"])))
        codes_at += (n + 255) // 256 * 256
        slot_at += 256


@pytest.mark.parametrize("fx,fw", [(E4M3, E4M3), (E4M3, E2M1), (E3M4, E3M0)])
def test_group_of_small_projections_dynamic_scale(fx, fw):
    """Shapes of the cross-attention key / value projections (616 x 768 -> 320 / 640 / 1280) plus ragged ones; 35
    problems, so the call spans two chunks of 32."""
    shapes = [(616, 768, 320), (616, 768, 640), (616, 768, 1280), (77, 768, 320), (130, 128, 65), (1, 16, 1), (200, 1280, 130)]
    shapes = (shapes * 5)[:35]
    ps = [make_problem(M, K, N, fx, fw, 9100 + 10 * i, with_bias=(i % 2 == 0)) for i, (M, K, N) in enumerate(shapes)]
    ws = run_group_dynamic(ps, fx, fw)
    check_group_dynamic(ps, fx, fw, ws)
    # the same problems one by one through fpq_gemm: these shapes take the same kernel there, so the sums agree bit for bit
    for p in ps[:7]:
        assert B.fpq_gemm_plan(p["M"], p["N"], p["K"])[0] in (B.FPQ_KERNEL_SMALL_TILE, B.FPQ_KERNEL_ROWS16)
        y1 = torch.full_like(p["y"], float("nan"))
        w1 = torch.empty(B.fpq_gemm_workspace_size(p["M"], p["N"], p["K"], 2), dtype=torch.uint8, device=DEV)
        B.fpq_gemm(p["x_t"], B.FPQ_X_FP32_DYNAMIC, fx, 0.0, None, p["packed"], fw, p["sw_t"], p["bias_t"], y1, p["M"], p["N"],
                   p["K"], B.FPQ_ACC_FP32, w1)
        torch.cuda.synchronize()
        if p["M"] > 16:
            assert torch.equal(y1, p["y"]), (p["M"], p["K"], p["N"])
        else:
            check_close(y1.cpu().numpy(), p["Y"], p["T"], what="single call")


@pytest.mark.parametrize("fw", [E4M3, E2M1])
def test_group_of_time_embedding_projections_one_launch(fw):
    """The residual blocks' time-embedding projections (8 x 1280 -> 320 / 640 / 1280): at most 16 rows each, so the
    whole group is one launch that also finds every problem's scale; bit-identical to the single-layer calls."""
    fx = E4M3
    shapes = [(8, 1280, 320), (8, 1280, 640), (8, 1280, 1280), (8, 320, 1280), (16, 1024, 48), (3, 64, 20)] * 4
    ps = [make_problem(M, K, N, fx, fw, 9500 + 10 * i, with_bias=(i % 3 == 0)) for i, (M, K, N) in enumerate(shapes)]
    ws = run_group_dynamic(ps, fx, fw)
    check_group_dynamic(ps, fx, fw, ws)
    for p in ps[:6]:
        y1 = torch.full_like(p["y"], float("nan"))
        w1 = torch.empty(B.fpq_gemm_workspace_size(p["M"], p["N"], p["K"], 2), dtype=torch.uint8, device=DEV)
        B.fpq_gemm(p["x_t"], B.FPQ_X_FP32_DYNAMIC, fx, 0.0, None, p["packed"], fw, p["sw_t"], p["bias_t"], y1, p["M"], p["N"],
                   p["K"], B.FPQ_ACC_FP32, w1)
        torch.cuda.synchronize()
        assert torch.equal(y1, p["y"]), (p["M"], p["K"], p["N"])


def test_group_on_codes_and_in_the_fp8_mfma_mode():
    fx, fw = E4M3, E4M3
    shapes = [(616, 768, 320), (300, 256, 96), (40, 2880, 160)]
    ps = [make_problem(M, K, N, fx, fw, 9800 + 10 * i, with_bias=True) for i, (M, K, N) in enumerate(shapes)]
    keep = [(dev(p["xq"]), dev(np.array([p["sx"]], dtype=np.float32))) for p in ps]
    for acc, rel in ((B.FPQ_ACC_FP32, 1e-5), (B.FPQ_ACC_FP8_MFMA, 7 * 2.0 ** -13)):
        for p in ps:
            p["y"].fill_(float("nan"))
        arr = B.gemm_problems([(xq_t, sx_t, p["packed"], p["sw_t"], p["bias_t"], p["y"], p["M"], p["N"], p["K"])
                               for p, (xq_t, sx_t) in zip(ps, keep)])
        assert B.fpq_gemm_grouped_workspace_size(arr, B.FPQ_X_CODES) == 0
        B.fpq_gemm_grouped(arr, B.FPQ_X_CODES, fx, fw, acc, None)
        torch.cuda.synchronize()
        for i, p in enumerate(ps):
            yh = p["y"].cpu().numpy()
            assert not np.isnan(yh).any()
            check_close(yh, p["Y"], p["T"], rel=rel, what="grouped codes problem %d acc %d" % (i, acc))


def test_grouped_call_in_a_graph_and_argument_checks():
    fx, fw = E4M3, E2M1
    ps = [make_problem(616, 768, 320, fx, fw, 9900 + 10 * i, with_bias=False) for i in range(3)]
    arr = B.gemm_problems([(p["x_t"], None, p["packed"], p["sw_t"], None, p["y"], p["M"], p["N"], p["K"]) for p in ps])
    ws = torch.empty(B.fpq_gemm_grouped_workspace_size(arr, 2), dtype=torch.uint8, device=DEV)
    B.fpq_gemm_grouped(arr, 2, fx, fw, B.FPQ_ACC_FP32, ws)
    torch.cuda.synchronize()
    eager = [p["y"].clone() for p in ps]
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            B.fpq_gemm_grouped(arr, 2, fx, fw, B.FPQ_ACC_FP32, ws)
    for rep in range(3):
        for p in ps:
            p["y"].fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for p, e in zip(ps, eager):
            assert torch.equal(p["y"], e), "replay %d" % rep
    L = B.lib()
    import ctypes as C
    assert L.fpq_gemm_grouped(arr, 3, 2, B.fmt(fx), B.fmt(fw), 0, None, 0, None) == -6          # dynamic form needs the workspace
    assert L.fpq_gemm_grouped(arr, 3, 1, B.fmt(fx), B.fmt(fw), 0, None, 0, None) == -8
    assert L.fpq_gemm_grouped(arr, 0, 2, B.fmt(fx), B.fmt(fw), 0, None, 0, None) == 0
    assert L.fpq_gemm_grouped(None, 3, 2, B.fmt(fx), B.fmt(fw), 0, None, 0, None) == -1
    bad = B.gemm_problems([(ps[0]["x_t"], None, ps[0]["packed"], ps[0]["sw_t"], None, ps[0]["y"], 616, 320, 760)])
    assert L.fpq_gemm_grouped(bad, 1, 2, B.fmt(fx), B.fmt(fw), 0, C.c_void_p(ws.data_ptr()), ws.numel(), None) == -5
