"""Pins of the oracle's 2-of-4 pruning rule for the structured-sparse weight operand (Section VI, "Sparsity"): brute
force over every group of four E2M1 codes, invariants, the literal tie and padding cases, and the vectorised form
against the loop."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2408_06995_amd import synth

E2M1, E4M3 = synth.E2M1, synth.E4M3


def eq5_magnitude(code, e, m, b):
    """Eq. (5) with the p = 0 row, written out here (not the oracle's decoder)."""
    f = code & ((1 << m) - 1)
    p = (code >> m) & ((1 << e) - 1)
    return (f / 2 ** m) * 2.0 ** (1 - b) if p == 0 else (1 + f / 2 ** m) * 2.0 ** (p - b)


def test_every_group_of_four_e2m1_codes_keeps_a_pair_of_largest_total_magnitude():
    """All 16^4 groups (signs included): at most two non-zeros survive, survivors are unchanged, and no other choice of
    two positions would have kept more magnitude (for 2-of-4 pruning that is the choice of least error in any norm)."""
    e, m, b, _ = E2M1
    groups = np.array(list(itertools.product(range(16), repeat=4)), dtype=np.uint8)        # [65536, 4] = [N, Cin]
    pruned, altered = oracle.prune_2of4_fast(groups, E2M1)
    mags = np.vectorize(lambda c: eq5_magnitude(int(c) & 7, e, m, b))(groups)
    kept = pruned != 0
    assert (kept.sum(axis=1) <= 2).all()
    assert np.array_equal(pruned[kept], groups[kept])                                       # survivors keep code and sign
    best = np.max([mags[:, [i, j]].sum(axis=1) for i, j in itertools.combinations(range(4), 2)], axis=0)
    got = np.where(kept, mags, 0.0).sum(axis=1)
    assert np.array_equal(got, best)
    nonzero = (mags != 0).sum(axis=1)
    pmags = np.vectorize(lambda c: eq5_magnitude(int(c) & 7, e, m, b))(pruned)
    assert np.array_equal(pmags[nonzero <= 2], mags[nonzero <= 2])                          # already sparse: values untouched
    assert altered == int((nonzero > 2).sum())
    again, altered2 = oracle.prune_2of4_fast(pruned, E2M1)
    assert np.array_equal(again, pruned) and altered2 == 0                                  # idempotent
    # the loop form on a slice of the same groups
    sub = groups[::97]
    p2, a2 = oracle.prune_2of4(sub, E2M1)
    assert np.array_equal(p2, pruned[::97]) and a2 == int((nonzero[::97] > 2).sum())


def test_ties_go_to_the_lower_channel_and_dropped_codes_become_plus_zero():
    one, two, neg_one = 2, 4, 2 | 8              # E2M1 (bias 1): code 2 = 1.0, code 4 = 2.0, sign bit = 8
    cases = [([one, one, one, one], [one, one, 0, 0]), ([0, two, two, two], [0, two, two, 0]),
             ([neg_one, one, two, one], [neg_one, 0, two, 0]), ([one, 0, 0, 8], [one, 0, 0, 0]),   # -0 counts as zero; not among the two kept, it becomes +0
             ([two, one, one, two], [two, 0, 0, two])]
    for src, want in cases:
        got, _ = oracle.prune_2of4(np.array([src], dtype=np.uint8), E2M1)
        assert got[0].tolist() == want, (src, got[0].tolist())


def test_groups_run_over_input_channels_per_tap_and_pad_with_zeros():
    rng = np.random.default_rng(4)
    w = rng.integers(0, 16, size=(3, 6, 3, 3), dtype=np.uint8)      # Cin = 6: groups (0..3) and (4, 5, -, -)
    pruned, altered = oracle.prune_2of4(w, E2M1)
    assert np.array_equal(pruned[:, 4:], w[:, 4:])                   # two real channels in the last group: nothing to drop
    for n in range(3):
        for kh in range(3):
            for kw in range(3):
                g, _ = oracle.prune_2of4(w[n:n + 1, :4, kh, kw], E2M1)
                assert np.array_equal(pruned[n, :4, kh, kw], g[0])
    f, a = oracle.prune_2of4_fast(w, E2M1)
    assert np.array_equal(f, pruned) and a == altered


@pytest.mark.parametrize("fmt", [E4M3, E2M1, synth.E3M0])
def test_vectorised_form_equals_the_loop_and_quantized_gaussians_are_mostly_sparse_already(fmt):
    w = synth.weights((24, 40), 77)
    wq, sw = oracle.pack_weights(w, fmt)
    a, na = oracle.prune_2of4(wq, fmt)
    b, nb = oracle.prune_2of4_fast(wq, fmt)
    assert np.array_equal(a, b) and na == nb
    assert ((b.reshape(24, 10, 4) & ((1 << (fmt[0] + fmt[1])) - 1)) != 0).sum(axis=2).max() <= 2
    # a layer on the pruned codes differs from the layer on the full codes exactly by the dropped products
    x = oracle.quantize(synth.activations((5, 40), 78), E4M3, 0.02)
    Y0, _ = oracle.gemm(x, E4M3, 0.02, wq, fmt, sw)
    Y1, _ = oracle.gemm(x, E4M3, 0.02, b, fmt, sw)
    dropped = wq.copy()
    dropped[b == wq] = 0
    Yd, _ = oracle.gemm(x, E4M3, 0.02, dropped, fmt, sw)
    assert np.allclose(Y0, Y1 + Yd, rtol=1e-12, atol=1e-12)
