"""Pins of the uniform integer quantizer's oracle (Eq. (4)) and of the integer layer: the equation's own properties,
brute force over the integer grid, hand cases, and numpy float64 matrix products of independently dequantized values."""
import numpy as np
import pytest

from oracle import uniform as U
from paper_2408_06995_amd import synth


@pytest.mark.parametrize("bits", [8, 4])
def test_scale_and_zero_point_follow_the_equation(bits):
    x = synth.activations((4096,), 11)
    s, z = U.params(x, bits)
    lo, hi = float(x.min()), float(x.max())
    assert abs(s - (hi - lo) / (2 ** bits - 1)) <= 2e-7 * s            # fp32 roundings of the range and the quotient
    assert z == -int(np.rint(np.float32(np.float32(lo) * np.float32(np.float32(1) / np.float32(s)))))
    assert 0 <= z <= 2 ** bits - 1                                      # data straddles zero: zero point inside the range
    q = U.quantize(x, bits, s, z)
    assert q.min() == 0 and q.max() == 2 ** bits - 1                    # min and max land on the end codes
    # hand cases: [0, 1, 2, 3] at 2 bits would be s = 1, z = 0; at 8 bits [−1, 0, 1.55]: s = 0.01, z = 100
    s2, z2 = U.params(np.array([-1.0, 0.0, 1.55], dtype=np.float32), 8)
    assert abs(s2 - 0.01) < 1e-8 and z2 == 100
    assert U.quantize(np.array([-1.0, 0.0, 1.55, 0.004, 0.006, -5.0, 9.0], dtype=np.float32), 8, s2, z2).tolist() == \
        [0, 100, 255, 100, 101, 0, 255]
    # all-positive data: the zero point leaves the code range, as the equation says
    s3, z3 = U.params(np.array([2.0, 3.0, 4.0], dtype=np.float32), 8)
    assert z3 == -255 and abs(s3 - 2.0 / 255) < 1e-9
    assert U.quantize(np.array([2.0, 4.0], dtype=np.float32), 8, s3, z3).tolist() == [0, 255]
    assert U.params(np.full(7, 3.5, dtype=np.float32), 8) == (1.0, -4)   # constant tensor: s = 1


@pytest.mark.parametrize("bits", [8, 4])
def test_codes_are_the_nearest_grid_point_by_brute_force(bits):
    rng = np.random.default_rng(bits)
    x = (rng.standard_normal(3000) * np.where(rng.random(3000) < 0.01, 20.0, 1.0)).astype(np.float32)
    s, z = U.params(x, bits)
    # probe beyond the range too, and exact ties
    probe = np.concatenate([x, x * np.float32(1.7), (np.arange(-5, 40) + 0.5).astype(np.float32) * np.float32(s)])
    q = U.quantize(probe, bits, s, z)
    r = np.float32(np.float32(1) / np.float32(s))
    y = (probe * r).astype(np.float32).astype(np.float64)               # the contract's fp32 quotient
    grid = np.arange(2 ** bits, dtype=np.float64) - z                   # (q - z) for every code
    d = np.abs(y[:, None] - grid[None, :])
    best = d.min(axis=1)
    assert np.array_equal(np.abs(y - (q.astype(np.float64) - z)), best)  # a nearest grid point (clamping included)
    tie = (d == best[:, None]).sum(axis=1) == 2                           # exact ties: the even integer n = q - z wins
    assert tie.any()
    assert (((q[tie].astype(np.int64) - z) % 2) == 0).all()
    inside = (probe >= x.min()) & (probe <= x.max())
    assert np.all(np.abs(probe[inside].astype(np.float64) - U.dequantize(q[inside], s, z)) <= 0.5 * s * (1 + 1e-5))
    assert np.all(np.diff(U.quantize(np.sort(probe), bits, s, z).astype(np.int64)) >= 0)   # monotone


def test_per_channel_weights_and_dequantize():
    w = synth.weights((12, 80), 3)
    for bits in (8, 4):
        q, s, z = U.pack_weights(w, bits)
        for n in range(12):
            sn, zn = U.params(w[n], bits)
            assert (s[n], z[n]) == (np.float32(sn), zn)
            assert np.array_equal(q[n], U.quantize(w[n], bits, sn, zn))
        assert np.all(np.abs(U.dequantize(q, s, z) - w) <= 0.5 * s[:, None] * (1 + 1e-5))


def test_integer_layer_equals_float64_products_and_a_hand_loop():
    rng = np.random.default_rng(2)
    x = synth.activations((9, 40), 5)
    w = synth.weights((7, 40), 6)
    sx, zx = U.params(x, 8)
    xq = U.quantize(x, 8, sx, zx)
    for bits in (8, 4):
        wq, sw, zw = U.pack_weights(w, bits)
        bias = rng.standard_normal(7).astype(np.float32)
        Y, T = U.gemm(xq, sx, zx, wq, sw, zw, bias)
        want = U.dequantize(xq, sx, zx) @ U.dequantize(wq, sw, zw).T + bias.astype(np.float64)[None, :]
        assert np.allclose(Y, want, rtol=1e-12, atol=1e-12)
        for m, n in ((0, 0), (8, 6), (4, 3)):
            acc = sum((int(xq[m, k]) - zx) * (int(wq[n, k]) - int(zw[n])) for k in range(40))
            assert Y[m, n] == float(np.float32(sx)) * float(sw[n]) * acc + float(bias[n])
            assert T[m, n] == float(np.float32(sx)) * float(sw[n]) * sum(abs((int(xq[m, k]) - zx) * (int(wq[n, k]) - int(zw[n])))
                                                                             for k in range(40))
        Yr, _ = U.gemm(xq, sx, zx, wq, sw, zw, bias, rows=[8, 2])
        assert np.array_equal(Yr, Y[[8, 2]])
        # the identity the matrix-unit form relies on: offsets c, d folded out with row sums
        c, d = 128, 8 if bits == 4 else 128
        a = xq.astype(np.int64) - c
        b = wq.astype(np.int64) - d
        zc, zd = zx - c, zw.astype(np.int64) - d
        I = a @ b.T
        folded = I - a.sum(axis=1)[:, None] * zd[None, :] - zc * b.sum(axis=1)[None, :] + 40 * zc * zd[None, :]
        assert np.array_equal(folded, (xq.astype(np.int64) - zx) @ (wq.astype(np.int64) - zw.astype(np.int64)[:, None]).T)
