"""Pins of the oracle's AutoFreeze score (Sec. 2.3) and Alg. 2 budget
reconciliation (App. "Hybrid Variants Algorithm") against the mathematics."""
import itertools
import math

import numpy as np
import pytest

import oracle


# ---------------------------------------------------------------- AutoFreeze
def test_norm_of_hand_made_updates():
    snap = np.zeros(2)
    assert oracle.autofreeze_sqnorm(np.array([3.0, 4.0]), snap) == 25.0                    # 3-4-5
    n, c = 1000, 0.25
    p = np.full(n, 1.0)
    assert oracle.autofreeze_sqnorm(p + c, p) == pytest.approx(n * c * c, rel=1e-15)         # ||c 1|| = |c| sqrt(n)
    # the update is what matters, not the parameters: shifting both leaves the norm alone
    rng = np.random.default_rng(1)
    a, b = rng.standard_normal(257), rng.standard_normal(257)
    assert oracle.autofreeze_sqnorm(a + 100.0, b + 100.0) == pytest.approx(oracle.autofreeze_sqnorm(a, b), rel=1e-12)
    assert oracle.autofreeze_sqnorm(a, b) == pytest.approx(oracle.autofreeze_sqnorm(b, a), rel=1e-15)   # symmetric
    assert oracle.autofreeze_sqnorm(a, a) == 0.0


def test_score_closed_forms():
    s = oracle.autofreeze_score
    assert s(4.0, 4.0) == 0.0                               # same norm: no change
    assert s(4.0, 1.0) == pytest.approx(0.5)                # norm 2 -> 1
    assert s(1.0, 4.0) == pytest.approx(1.0)                # norm 1 -> 2: |1 - 2| / 1
    assert s(9.0, 0.0) == pytest.approx(1.0)                # stopped moving altogether
    assert s(0.0, 0.0) == 0.0 and s(0.0, 1.0) == math.inf   # the conventions for a zero denominator
    # scale invariance: both norms times c leave the score alone
    assert s(4.0 * 49, 1.0 * 49) == pytest.approx(s(4.0, 1.0))


def test_threshold_is_numpys_nearest_rank_percentile():
    rng = np.random.default_rng(7)
    for L in (1, 2, 5, 14, 28):
        sc = rng.random(L)
        for P in (10.0, 50.0, 80.0, 100.0):
            tau = np.percentile(sc, P, method="inverted_cdf")
            qualifies = sc <= tau
            expect = np.zeros(L, np.uint8)
            l = 0
            while l < L and qualifies[l]:
                expect[l] = 1
                l += 1
            assert np.array_equal(oracle.autofreeze_select(sc, 0, P), expect), (L, P)


def test_frozen_set_is_a_prefix_and_grows_with_the_percentile():
    for L in range(1, 6):
        for perm in itertools.permutations(range(L)):
            sc = [float(v) for v in perm]
            prev = -1
            for P in (0.0, 20.0, 40.0, 60.0, 80.0, 100.0):
                for k0 in range(L + 1):
                    m = oracle.autofreeze_select(sc, k0, P)
                    n = int(m.sum())
                    assert np.array_equal(m, np.r_[np.ones(n, np.uint8), np.zeros(L - n, np.uint8)])   # a prefix
                    assert n >= k0                                                                     # never thaws
                n0 = int(oracle.autofreeze_select(sc, 0, P).sum())
                assert n0 >= prev
                prev = n0
            # P = 100: every trained layer qualifies, so everything freezes; P = 0: nothing does
            assert oracle.autofreeze_select(sc, 0, 100.0).sum() == L
            assert oracle.autofreeze_select(sc, 0, 0.0).sum() == 0


def test_a_layer_behind_an_unstable_one_stays_trained():
    # layer 0 unstable (largest change) blocks the prefix although layers 1.. are stable
    assert oracle.autofreeze_select([0.9, 0.1, 0.1, 0.1, 0.1], 0, 80.0).sum() == 0
    # once layer 0 is frozen the next check can take the rest of the lower 80 %: 4 trained, rank ceil(3.2) = 4
    assert list(oracle.autofreeze_select([0.0, 0.1, 0.1, 0.1, 0.5], 1, 80.0)) == [1, 1, 1, 1, 1]
    assert list(oracle.autofreeze_select([0.0, 0.1, 0.1, 0.1, 0.5], 1, 75.0)) == [1, 1, 1, 1, 0]


# -------------------------------------------------------------------- Alg. 2
def test_keyed_permutation_is_invertible():
    rng = np.random.default_rng(3)
    x = np.r_[np.arange(0, 70000, dtype=np.uint64), rng.integers(0, 1 << 32, 50000, dtype=np.uint64),
              np.array([(1 << 32) - 1, 1 << 31, 65535, 65536], dtype=np.uint64)]
    for seed in (0, 1, 0xDEADBEEFCAFEF00D, (1 << 64) - 1):
        y = oracle.perm32(x, seed)
        assert np.array_equal(oracle.perm32_inverse(y, seed).astype(np.uint64), x)
    # an inverse exists => no two indices share a key; check it outright on a full 2^16 block
    y = oracle.perm32(np.arange(1 << 16, dtype=np.uint64) + (5 << 16), 99)
    assert np.unique(y).size == 1 << 16
    # different seeds give different permutations
    assert not np.array_equal(oracle.perm32(x[:1000], 1), oracle.perm32(x[:1000], 2))


def _random_base(rng, numel, density):
    return [(rng.random(n) < density).astype(np.uint8) for n in numel]


@pytest.mark.parametrize("density", [0.0, 0.2, 0.5, 0.9, 1.0])
def test_budget_is_met_exactly_and_the_base_mask_is_respected(density):
    rng = np.random.default_rng(int(density * 100) + 5)
    numel = [1, 33, 1000, 4097, 31]
    N = sum(numel)
    base = _random_base(rng, numel, density)
    base_flat = np.concatenate(base)
    c = int(base_flat.sum())
    for r in (0.0, 0.1, 0.33, 0.5, 0.8, 1.0):
        nf = math.floor(r * N)
        new, count = oracle.reconcile_mask(base, numel, nf, seed=1234)
        new_flat = np.concatenate(new)
        assert count == c
        assert int(new_flat.sum()) == nf                                   # ||I||_1 = N_freeze, exactly
        assert [len(a) for a in new] == numel
        if c <= nf:
            assert np.all(new_flat >= base_flat)                           # only additions
        if c >= nf:
            assert np.all(new_flat <= base_flat)                           # only removals
    same, _ = oracle.reconcile_mask(base, numel, c, seed=1)
    assert np.array_equal(np.concatenate(same), base_flat)                 # budget already met: untouched


def test_selection_is_the_lowest_keys_among_the_candidates():
    rng = np.random.default_rng(11)
    numel = [50, 77]
    base = _random_base(rng, numel, 0.3)
    flat = np.concatenate(base)
    c, N = int(flat.sum()), sum(numel)
    seed = 42
    keys = oracle.perm32(np.arange(N), seed)
    # add: the added indices are zeros of the base mask and every zero left out has a larger key
    new = np.concatenate(oracle.reconcile_mask(base, numel, c + 20, seed)[0])
    added = np.flatnonzero((new == 1) & (flat == 0))
    left = np.flatnonzero((new == 0) & (flat == 0))
    assert added.size == 20 and keys[added].max() < keys[left].min()
    # remove: the dropped indices are ones of the base mask and every one that was kept has a larger key
    new = np.concatenate(oracle.reconcile_mask(base, numel, c - 10, seed)[0])
    dropped = np.flatnonzero((new == 0) & (flat == 1))
    kept = np.flatnonzero((new == 1) & (flat == 1))
    assert dropped.size == 10 and keys[dropped].max() < keys[kept].min()
    # same seed, same answer; another seed, another subset
    again = np.concatenate(oracle.reconcile_mask(base, numel, c + 20, seed)[0])
    other = np.concatenate(oracle.reconcile_mask(base, numel, c + 20, seed + 1)[0])
    assert np.array_equal(again, np.concatenate(oracle.reconcile_mask(base, numel, c + 20, seed)[0]))
    assert not np.array_equal(again, other)


def test_every_candidate_is_equally_likely_over_seeds():
    # chi-square of the inclusion counts of 64 candidates, 16 drawn, over 4000 seeds
    n, m, trials = 64, 16, 4000
    base = [np.zeros(n, np.uint8)]
    hits = np.zeros(n)
    for seed in range(trials):
        hits += oracle.reconcile_mask(base, [n], m, seed * 2654435761 + 17)[0][0]
    expect = trials * m / n
    # inclusion indicators have variance p(1-p) per trial
    chi2 = float(((hits - expect) ** 2).sum() / (trials * (m / n) * (1 - m / n)))
    assert 30.0 < chi2 < 110.0, chi2          # 63 degrees of freedom: mean 63, sd ~11
    # pairs of neighbours are not drawn together more often than chance: P(both) = m(m-1)/(n(n-1))
    both = 0
    for seed in range(trials):
        b = oracle.reconcile_mask(base, [n], m, seed * 40503 + 1)[0][0]
        both += int((b[:-1] & b[1:]).sum())
    p_both = m * (m - 1) / (n * (n - 1))
    assert abs(both / (trials * (n - 1)) - p_both) < 0.01


def test_bit_packing_round_trip():
    rng = np.random.default_rng(2)
    for n in (1, 31, 32, 33, 1000):
        b = (rng.random(n) < 0.5).astype(np.uint8)
        w = oracle.pack_bits(b)
        assert w.dtype == np.dtype("<u4") and w.size == (n + 31) // 32
        assert np.array_equal(oracle.unpack_bits(w, n), b)
        assert (int(w[0]) & 1) == int(b[0])            # LSB first


# ------------------------------------------------------- sub-tensor freezing
def test_row_block_draw_fills_the_budget_to_within_one_unit():
    shapes = [(2048, 2048), (2048, 512), (2048, 512), (2048, 2048), (2048, 8192), (2048, 8192), (8192, 2048)] * 2
    P = sum(k * n for k, n in shapes)
    smallest = 256 * 512
    prev = None
    for r in (0.0, 0.1, 0.25, 0.5, 0.75, 0.9, 1.0):
        masks, frozen = oracle.select_row_blocks(shapes, 256, r, seed=7)
        budget = math.floor(r * P + 1e-9)
        assert frozen == sum(int(m.sum()) * 256 * n for m, (k, n) in zip(masks, shapes))
        assert frozen <= budget
        untaken = [256 * n for m, (k, n) in zip(masks, shapes) for f in m if not f]
        assert not untaken or budget - frozen < min(untaken)           # no unit left that would still fit
        assert budget - frozen < 256 * 8192                            # hence within one (largest) unit
        assert [len(m) for m in masks] == [k // 256 for k, _ in shapes]
    assert oracle.select_row_blocks(shapes, 256, 1.0, 3)[1] == P and oracle.select_row_blocks(shapes, 256, 0.0, 3)[1] == 0
    a, _ = oracle.select_row_blocks(shapes, 256, 0.5, 11)
    b, _ = oracle.select_row_blocks(shapes, 256, 0.5, 11)
    c, _ = oracle.select_row_blocks(shapes, 256, 0.5, 12)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert any(not np.array_equal(x, y) for x, y in zip(a, c))
    assert smallest > 0


def test_row_block_draw_treats_equal_units_alike():
    shapes = [(1024, 64)] * 2                       # 32 equal units of 32 rows
    hits = np.zeros(64)
    trials = 3000
    for seed in range(trials):
        masks, frozen = oracle.select_row_blocks(shapes, 32, 0.25, seed * 7919 + 3)
        assert frozen == 16 * 32 * 64               # equal units: the budget is met exactly
        hits += np.concatenate(masks)
    chi2 = float(((hits - trials / 4) ** 2).sum() / (trials * 0.25 * 0.75))
    assert 30.0 < chi2 < 110.0, chi2                # 63 degrees of freedom


def test_backward_with_row_blocks_equals_the_full_backward_on_unfrozen_rows():
    rng = np.random.default_rng(5)
    shapes, T, br = [(8, 6), (12, 5), (4, 7)], 9, 4
    W = [rng.standard_normal(s) for s in shapes]
    X = [rng.standard_normal((T, k)) for k, n in shapes]
    dY = [rng.standard_normal((T, n)) for k, n in shapes]
    full_dX = [np.zeros((T, k)) for k, n in shapes]
    full_dW = [np.zeros(s) for s in shapes]
    oracle.stage_backward(shapes, T, W, X, dY, [0, 0, 0], full_dX, full_dW)
    assert all(np.allclose(a, x.T @ g, atol=1e-12) for a, x, g in zip(full_dW, X, dY))      # the textbook product
    canary = [np.full(s, np.nan) for s in shapes]
    for a in canary:
        a.view(np.uint64)[...] = 0x7FF8000000000ABC                                          # NaN with a payload
    row_masks = [np.array([1, 0], np.uint8), np.array([0, 1, 0], np.uint8), None]
    dX = [np.zeros((T, k)) for k, n in shapes]
    dW = [c.copy() for c in canary]
    oracle.stage_backward_blocks(shapes, T, W, X, dY, [0, 0, 0], row_masks, br, dX, dW)
    for l, (k, n) in enumerate(shapes):
        assert np.array_equal(dX[l], full_dX[l])                                              # dX does not depend on the masks
        rm = row_masks[l] if row_masks[l] is not None else np.zeros(k // br, np.uint8)
        for b, f in enumerate(rm):
            rows = slice(b * br, (b + 1) * br)
            if f:
                assert dW[l][rows].tobytes() == canary[l][rows].tobytes()                     # frozen rows: not a bit changed
            else:
                assert np.array_equal(dW[l][rows], full_dW[l][rows])
    # accumulation adds onto what is there; a frozen tensor overrides its row mask
    acc = [np.ones(s) for s in shapes]
    oracle.stage_backward_blocks(shapes, T, W, X, dY, [0, 1, 0], row_masks, br, dX, acc, accumulate=True)
    assert np.array_equal(acc[1], np.ones(shapes[1]))
    assert np.allclose(acc[0][4:], 1.0 + full_dW[0][4:]) and np.array_equal(acc[0][:4], np.ones((4, 6)))
    assert np.allclose(acc[2], 1.0 + full_dW[2])
    # all blocks frozen == tensor frozen; element mask of a row mask
    em = oracle.row_blocks_to_elem_mask((8, 6), 4, [1, 0])
    assert em.tolist() == [1] * 24 + [0] * 24
