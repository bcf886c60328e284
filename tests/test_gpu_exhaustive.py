"""All 2^32 fp32 bit patterns through the activation quantizer (Eq. (6), (8), (9)) on the GPU against the oracle, for the
hardware-range E4M3 format at scale 1 and at a scale that is not a power of two: every exponent, every mantissa,
denormals, both zeros and both infinities.  NaN patterns are outside the quantizer's contract and are replaced by
zeros on both sides."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth
from gpu_util import DEV

pytestmark = pytest.mark.gpu

CHUNK = 1 << 25
PARTS = 8                      # the sweep is cut into parts so that no single test runs for minutes
SEEN = {}                      # scale -> how often each code came out, summed over the parts that have run


@pytest.mark.parametrize("part", range(PARTS))
@pytest.mark.parametrize("scale", [1.0, 0.7331])
def test_quantize_every_fp32_bit_pattern(scale, part):
    f = synth.E4M3
    scale = float(np.float32(scale))
    codes = torch.empty(CHUNK, dtype=torch.uint8, device=DEV)
    seen = SEEN.setdefault(scale, np.zeros(257, dtype=np.int64))
    per_part = (1 << 32) // PARTS
    for lo in range(part * per_part, (part + 1) * per_part, CHUNK):
        bits = np.arange(lo, lo + CHUNK, dtype=np.uint32)
        nan = ((bits & 0x7F800000) == 0x7F800000) & ((bits & 0x007FFFFF) != 0)
        bits[nan] = 0
        x = bits.view(np.float32)
        B.fpq_quantize(torch.from_numpy(x).to(DEV), f, scale, None, codes)
        torch.cuda.synchronize()
        got = codes.cpu().numpy()
        want = oracle.quantize(x, f, scale)
        if not np.array_equal(got, want):
            bad = np.flatnonzero(got != want)
            raise AssertionError("scale %r: %d codes differ in the chunk at 0x%08x, first at bit pattern 0x%08x (gpu %d, "
                                 "oracle %d)" % (scale, bad.size, lo, int(bits[bad[0]]), int(got[bad[0]]), int(want[bad[0]])))
        seen[:256] += np.bincount(got, minlength=256)
    seen[256] += 1
    if seen[256] == PARTS:
        # all parts ran: every code of the format was produced except the two all-ones magnitudes, which
        # (4, 3, 7, 448) does not have
        assert seen[:256].sum() == 1 << 32
        assert np.all(seen[:256][np.arange(256) & 0x7F != 0x7F] > 0) and seen[0x7F] == 0 and seen[0xFF] == 0
