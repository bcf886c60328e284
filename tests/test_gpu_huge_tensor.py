"""A tensor of more than 2^32 elements (17 GB of fp32) through every pass that takes an element count: the
encoding / bias search, absmax, the quantizer in both code layouts, and the zero count.  The tensor is a seeded
block of 2^22 values repeated 1025 times on the device plus a ragged tail of 5, so the oracle's results for the
block and the tail give the expected result of the whole, exactly for codes and counts."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV, dev

pytestmark = pytest.mark.gpu

T, REPS, TAIL = 1 << 22, 1025, 5
N = T * REPS + TAIL


def test_more_than_two_to_the_32_elements():
    assert N > 2 ** 32
    base = synth.activations((T,), 96)
    tail = (synth.activations((TAIL,), 97) * np.float32(0.01)).astype(np.float32)   # stays below the block's maximum
    x = torch.empty(N, dtype=torch.float32, device=DEV)
    x[:T * REPS].view(REPS, T).copy_(dev(base).view(1, T).expand(REPS, T))
    x[T * REPS:] = dev(tail)
    small = np.concatenate([base, tail])

    # ---- encoding / bias search: the mean error of the whole is that of block + tail up to the tail's weight
    enc, J = [(2, 5), (3, 4), (4, 3), (5, 2)], 16
    print("search", flush=True)
    mse = torch.full((len(enc) * J,), float("nan"), dtype=torch.float32, device=DEV)
    res = torch.zeros(40, dtype=torch.uint8, device=DEV)
    ws = torch.empty(B.fpq_search_workspace_size(N, len(enc), J), dtype=torch.uint8, device=DEV)
    B.fpq_search_format(x, enc, J, mse, res, ws)
    torch.cuda.synchronize()
    got = mse.cpu().numpy().reshape(len(enc), J)
    want_block, _ = oracle.search(base, enc, J)
    want_small, _ = oracle.search(small, enc, J)
    assert oracle.absmax(small) == oracle.absmax(base)
    sse_tail = want_small * small.size - want_block * T
    want = (want_block * T * REPS + sse_tail) / N
    assert np.all(np.abs(got - want) <= 1e-4 * want), float(np.max(np.abs(got - want) / want))
    r = B.search_result(res)
    assert want[r.encoding, r.bias_index] <= want.min() * (1 + 2e-4)

    # ---- absmax: the maximum sits in the tail, beyond element 2^32
    print("absmax", flush=True)
    big = np.float32(3.0) * np.float32(oracle.absmax(base))
    x[N - 3] = float(big)
    tail[TAIL - 3] = big
    ws = torch.empty(B.fpq_absmax_workspace_size(N) // 4 + 1, dtype=torch.float32, device=DEV)
    out = torch.empty(2, dtype=torch.float32, device=DEV)
    B.fpq_absmax(x, 448.0, out[0:1], out[1:2], ws)
    torch.cuda.synchronize()
    sx = oracle.scale_from_absmax(float(big), 448.0)
    assert out.cpu().numpy().tolist() == [float(big), float(np.float32(sx))]

    # ---- quantizer, one code per byte and two per byte (N is odd: the last byte's high nibble stays 0)
    zc = torch.zeros(1, dtype=torch.int64, device=DEV)
    zws = torch.empty(B.fpq_count_zeros_workspace_size(N), dtype=torch.uint8, device=DEV)
    for f in (synth.E4M3, synth.E2M1):
        s = oracle.scale_from_absmax(float(big), f[3])
        cb, ct = oracle.quantize(base, f, s), oracle.quantize(tail, f, s)
        four = B.fpq_code_bytes(N, f) != N
        print("quantize", f, flush=True)
        codes = torch.full((B.fpq_code_bytes(N, f) + 16,), 0xA5, dtype=torch.uint8, device=DEV)
        B.fpq_quantize(x, f, s, None, codes)
        torch.cuda.synchronize()
        nb = B.fpq_code_bytes(N, f)
        assert bool((codes[nb:] == 0xA5).all())
        if four:
            eb, et = dev(oracle.pack4(cb)), dev(oracle.pack4(ct))
            per = T // 2
        else:
            eb, et = dev(cb), dev(ct)
            per = T
        assert bool((codes[:per * REPS].view(REPS, per) == eb.view(1, per)).all())
        assert torch.equal(codes[per * REPS:nb], et)
        # ---- zero count on those codes
        B.fpq_count_zeros(codes, B.FPQ_X_CODES, N, f, zc, zws)
        torch.cuda.synchronize()
        assert int(zc.item()) == REPS * oracle.count_zero_codes(cb, f) + oracle.count_zero_codes(ct, f)
        del codes
    # ---- and on the fp32 values themselves
    x[5] = 0.0
    x[N - 1] = -0.0
    B.fpq_count_zeros(x, B.FPQ_X_FP32, N, None, zc, zws)
    torch.cuda.synchronize()
    zb = oracle.count_zeros(base)
    assert int(zc.item()) == REPS * zb + oracle.count_zeros(tail[:-1]) + 1 + (0 if base[5] == 0 else 1)
