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
