"""Encoding / bias search (Section V-A, Algorithm 1): the HIP reduction against the oracle's 444 quantizer passes."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import oracle
from paper_2408_06995_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

FP8 = [(2, 5), (3, 4), (4, 3), (5, 2)]
FP4 = [(1, 2), (2, 1)]
# per-candidate error: one fp32 rounding of each difference (2^-24), fp32 sums of <= 512 non-negative terms per
# wavefront and round (<= 512 * 2^-24 relative), fp32 adds across rounds and waves, fp64 across blocks
REL = 1e-4


def run_search(x, encodings, J):
    from paper_2408_06995_amd import binding as B
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    mse = torch.full((len(encodings) * J,), float("nan"), dtype=torch.float32, device="cuda")
    res = torch.zeros(40, dtype=torch.uint8, device="cuda")
    ws = torch.empty(B.fpq_search_workspace_size(x.size, len(encodings), J), dtype=torch.uint8, device="cuda")
    B.fpq_search_format(xd, encodings, J, mse, res, ws)
    torch.cuda.synchronize()
    return mse.cpu().numpy().reshape(len(encodings), J), B.search_result(res)


def check(x, encodings, J):
    got, r = run_search(x, encodings, J)
    want, best = oracle.search(x, encodings, J)
    assert np.all(np.abs(got - want) <= REL * want + 1e-30), float(np.max(np.abs(got - want) / (want + 1e-30)))
    # the argmin is a floating-point decision: the chosen candidate must be a minimum up to the error bound
    assert want[r.encoding, r.bias_index] <= want.min() * (1 + 2 * REL)
    if want.size > 1 and want[best] * (1 + 2 * REL) < np.partition(want.reshape(-1), 1)[1]:   # unique beyond the bound
        assert (r.encoding, r.bias_index) == best
    e, m = encodings[r.encoding]
    assert (r.ebits, r.mbits, r.int_bias) == (e, m, 1 << (e - 1))
    absmax = oracle.absmax(x)
    cj = oracle.search_candidate(absmax, r.bias_index, J)
    assert r.maxval == np.float32(cj) and r.scale == np.float32(oracle.search_scale(e, m, cj))
    assert abs(r.mse - want[r.encoding, r.bias_index]) <= REL * want[r.encoding, r.bias_index] + 1e-30
    # Eq. (7) at the reported real-valued bias gives back the max value
    assert abs((2 - 2.0 ** -m) * 2.0 ** (2 ** e - r.real_bias - 1) - cj) <= 1e-5 * cj
    return r


@pytest.mark.parametrize("encodings,J", [(FP8, 111), (FP4, 111), (FP8, 7), ([(4, 3)], 1), (FP8 + FP4, 128)])
@pytest.mark.parametrize("n", [1, 5, 2047, 2048, 40000])
def test_search_matches_oracle_small(encodings, J, n):
    check(synth.activations((n,), 300 + n), encodings, J)


def test_search_activation_and_weight_tensors():
    check(synth.activations((1, 320, 64, 64), 2000).reshape(-1), FP8, 111)      # configuration 2's activations
    check(synth.weights((320, 320, 3, 3), 2500).reshape(-1), FP4, 111)          # and weights
    # ragged length and a pointer that is not 16-byte aligned
    xd = torch.from_numpy(np.ascontiguousarray(synth.activations(((1 << 20) + 4,), 9))).cuda()[1:]
    from paper_2408_06995_amd import binding as B
    mse = torch.empty(4 * 111, dtype=torch.float32, device="cuda")
    res = torch.zeros(40, dtype=torch.uint8, device="cuda")
    ws = torch.empty(B.fpq_search_workspace_size(xd.numel(), 4, 111), dtype=torch.uint8, device="cuda")
    B.fpq_search_format(xd, FP8, 111, mse, res, ws)
    torch.cuda.synchronize()
    want, _ = oracle.search(xd.cpu().numpy(), FP8, 111)
    assert np.all(np.abs(mse.cpu().numpy().reshape(4, 111) - want) <= REL * want)


def test_search_degenerate_tensors():
    r = check(np.zeros(1000, np.float32), FP8, 111)
    assert (r.encoding, r.bias_index, r.mse) == (0, 0, 0.0)
    s = np.float32(0.37)
    x = (np.array([0, .5, 1, 1.5, 2, 3, 4, 6] * 50, np.float32) * s * np.tile([1, -1], 200)).astype(np.float32)
    r = check(x, FP4, 111)
    assert (r.encoding, r.bias_index, r.mse) == (1, 110, 0.0)       # the grid the data lies on, found exactly


def test_search_result_feeds_the_quantizer():
    """The (format, scale) the search reports, given to fpq_quantize, reproduces the candidate's error."""
    from paper_2408_06995_amd import binding as B
    x = synth.activations((50000,), 4)
    r = check(x, FP8, 111)
    fmt = (r.ebits, r.mbits, r.int_bias, 0.0)
    xd = torch.from_numpy(x).cuda()
    codes = torch.empty(x.size, dtype=torch.uint8, device="cuda")
    B.fpq_quantize(xd, fmt, r.scale, None, codes)
    deq = torch.empty(x.size, dtype=torch.float32, device="cuda")
    B.fpq_dequantize(codes, fmt, r.scale, deq)
    torch.cuda.synchronize()
    err = np.mean((x.astype(np.float64) - deq.cpu().numpy().astype(np.float64)) ** 2)
    assert abs(err - r.mse) <= 1e-4 * r.mse
