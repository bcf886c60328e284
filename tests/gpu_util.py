"""Helpers of the GPU parity tests: run a layer through the C ABI (via the binding) and through the
CPU oracle on the same host-generated inputs."""
import numpy as np
import torch

import oracle
from paper_2408_06995_amd import binding as B

DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_absmax_scale(x_t, maxval):
    ws = torch.zeros(max(2, B.fpq_absmax_workspace_size(x_t.numel()) // 4), dtype=torch.float32, device=DEV)
    out = torch.empty(2, dtype=torch.float32, device=DEV)
    B.fpq_absmax(x_t, maxval, out[0:1], out[1:2], ws)
    return out


def gpu_quantize(x_np, f, scale=None, scale_dev=None):
    x_t = dev(x_np)
    codes = torch.empty(B.fpq_code_bytes(x_t.numel(), f), dtype=torch.uint8, device=DEV)
    B.fpq_quantize(x_t, f, 0.0 if scale is None else scale, scale_dev, codes)
    torch.cuda.synchronize()
    return codes.cpu().numpy()


def gpu_pack(w_np, fw, mask_np=None, scale_np=None, want_codes=True):
    w_t = dev(w_np)
    N, Cin = w_np.shape[0], w_np.shape[1]
    kh, kw = (w_np.shape[2], w_np.shape[3]) if w_np.ndim == 4 else (1, 1)
    packed = torch.empty(B.fpq_packed_size(N, Cin, kh, kw, fw), dtype=torch.uint8, device=DEV)
    sw = torch.empty(N, dtype=torch.float32, device=DEV)
    codes = torch.empty(w_np.size, dtype=torch.uint8, device=DEV) if want_codes else None
    B.fpq_pack_weights(w_t, fw, None if scale_np is None else dev(scale_np), None if mask_np is None else dev(mask_np),
                       packed, sw, codes)
    torch.cuda.synchronize()
    return packed, sw, (codes.cpu().numpy().reshape(w_np.shape) if want_codes else None)


def check_close(y_gpu, Y, T, rel=1e-5, abs_=1e-6, what=""):
    """|gpu - oracle| <= rel * sum_k |a_k b_k| + abs per element."""
    err = np.abs(y_gpu.astype(np.float64) - Y)
    tol = rel * T + abs_
    bad = err > tol
    assert not bad.any(), "%s: %d of %d outside tolerance, worst err/tol %.3g" % (
        what, int(bad.sum()), bad.size, float((err / tol).max()))
    return float((err / tol).max())


def oracle_linear_inputs(x, w, h, fx, fw):
    sx = oracle.scale_from_absmax(oracle.absmax(x), fx[3])
    xq = oracle.quantize(x, fx, sx)
    wq, sw = oracle.pack_weights(w, fw, h)
    return sx, xq, wq, sw
