"""GPU parity of the AutoFreeze norms (Sec. 2.3) and of the Alg. 2 budget
reconciliation (App. "Hybrid Variants Algorithm") against the oracle.
Bounds: squared norms within 1e-12 relative (fp64 sums of exact differences;
only the order of summation differs); snapshots, masks, counts and the largest
key drawn bit-exact."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2602_05754_amd as tf

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = tf.Context(0)
    yield c
    c.close()


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


# ---------------------------------------------------------------- AutoFreeze
@pytest.mark.parametrize("update", [True, False])
def test_autofreeze_norms_and_snapshot(ctx, update):
    rs = np.random.default_rng(260205754 + int(update))
    numel = [1, 3, 4096, 4097, 5 * 4096 + 1234, 256 * 688, 100003]     # one element ... several blocks and ragged tails
    p = [_f32(rs.standard_normal(n) * 0.02) for n in numel]
    snap = [_f32(a + rs.standard_normal(a.size) * 1e-4) for a in p]
    mask = np.zeros(len(numel), np.uint8)
    mask[2] = 1                                                       # one tensor skipped
    dp = [torch.from_numpy(a).cuda() for a in p]
    ds = [torch.from_numpy(a).cuda() for a in snap]
    out = torch.full((len(numel),), -7.0, dtype=torch.float64, device="cuda")
    tf.tf_autofreeze_norms(ctx, numel, dp, ds, out, tensor_freeze_mask=mask, update_snapshot=update)
    got = out.cpu().numpy()
    for i, n in enumerate(numel):
        if mask[i]:
            assert got[i] == -7.0                                      # skipped: untouched
            assert np.array_equal(ds[i].cpu().numpy(), snap[i])
            continue
        ref = oracle.autofreeze_sqnorm(p[i], snap[i])
        assert got[i] == pytest.approx(ref, rel=1e-12), (i, n)
        assert np.array_equal(ds[i].cpu().numpy(), p[i] if update else snap[i])      # bit-exact snapshot
        assert np.array_equal(dp[i].cpu().numpy(), p[i])                             # parameters only read
    if update:      # a second check right away sees no movement at all
        tf.tf_autofreeze_norms(ctx, numel, dp, ds, out, tensor_freeze_mask=mask, update_snapshot=True)
        got2 = out.cpu().numpy()
        assert all(got2[i] == 0.0 for i in range(len(numel)) if not mask[i])


def test_autofreeze_norms_with_more_tensors_than_one_launch_holds(ctx):
    """75 tensors need three launches of the norm pass; the per-tensor sums are gathered through
    slots that every launch must leave zero for the next one (also for the optimizer's score sums,
    which share them).  Sizes from one element to many one-wave blocks per slot."""
    rs = np.random.default_rng(260205754 + 77)
    numel = [int(n) for n in rs.integers(1, 3000, size=72)] + [64 * 512 * 3 + 5, 700001, 2]
    p = [_f32(rs.standard_normal(n) * 0.02) for n in numel]
    snap = [_f32(a + rs.standard_normal(a.size) * 1e-4) for a in p]
    mask = np.zeros(len(numel), np.uint8)
    mask[[5, 40, 73]] = 1
    dp = [torch.from_numpy(a).cuda() for a in p]
    ds = [torch.from_numpy(a).cuda() for a in snap]
    out = torch.full((len(numel),), -7.0, dtype=torch.float64, device="cuda")
    for rep in range(2):            # the second call finds the slots as the first left them
        tf.tf_autofreeze_norms(ctx, numel, dp, ds, out, tensor_freeze_mask=mask, update_snapshot=False)
        got = out.cpu().numpy()
        for i, n in enumerate(numel):
            if mask[i]:
                assert got[i] == -7.0
            else:
                assert got[i] == pytest.approx(oracle.autofreeze_sqnorm(p[i], snap[i]), rel=1e-12), (rep, i, n)
    # the optimizer's score sums go through the same slots: still exact after the norm passes
    n = 3000
    E = _f32(rs.standard_normal(n) * 1e-5)
    A = _f32(np.abs(rs.standard_normal(n)) * 1e-4)
    d = _f32(rs.standard_normal(n) * 1e-5)
    dE, dA, dd = (torch.from_numpy(x.copy()).cuda() for x in (E, A, d))
    sums = torch.zeros(2, dtype=torch.float64, device="cuda")
    tf.tf_stability_update(ctx, [n], [dd], [dE], [dA], 0.99, score_sums=sums)
    E64, A64 = E.astype(np.float64), A.astype(np.float64)
    oracle.stability_update(d.astype(np.float64), E64, A64, 0.99)
    assert sums.cpu().numpy() == pytest.approx(np.array(oracle.score_sums(E64, A64)), rel=1e-5)


def test_autofreeze_check_sequence_matches_the_oracle_rule(ctx):
    """Three checks of a 14-layer stage whose early layers move less and less: norms -> scores ->
    prefix selection, every step against the oracle."""
    rs = np.random.default_rng(99)
    L = 14
    numel = [256 * 256] * 8 + [256 * 688] * 6
    p = [_f32(rs.standard_normal(n) * 0.02) for n in numel]
    dp = [torch.from_numpy(a.copy()).cuda() for a in p]
    ds = [torch.from_numpy(a.copy()).cuda() for a in p]
    host_snap = [a.copy() for a in p]
    out = torch.zeros(L, dtype=torch.float64, device="cuda")
    sq_prev = sq_prev_ref = None
    frozen = 0
    for check in range(3):
        for l in range(L):                                            # the interval's cumulative update
            scale = 1e-3 * (1.0 if l >= 5 else 0.5 ** check) * (1.0 + 0.3 * rs.random())
            p[l] = _f32(p[l] + rs.standard_normal(numel[l]) * scale)
            dp[l].copy_(torch.from_numpy(p[l]))
        tf.tf_autofreeze_norms(ctx, numel, dp, ds, out)
        sq = out.cpu().numpy().copy()
        sq_ref = np.array([oracle.autofreeze_sqnorm(p[l], host_snap[l]) for l in range(L)])
        assert np.allclose(sq, sq_ref, rtol=1e-12, atol=0)
        host_snap = [a.copy() for a in p]
        if sq_prev is not None:
            sc = tf.tf_autofreeze_scores(sq_prev, sq)
            sc_ref = np.array([oracle.autofreeze_score(a, b) for a, b in zip(sq_prev_ref, sq_ref)])
            assert np.allclose(sc, sc_ref, rtol=1e-9)
            m = tf.tf_autofreeze_select(sc, frozen, 80.0)
            assert np.array_equal(m, oracle.autofreeze_select(sc_ref, frozen, 80.0))
            frozen = int(m.sum())
        sq_prev, sq_prev_ref = sq, sq_ref
    assert frozen >= 1                                                 # the slowing prefix did get frozen


# -------------------------------------------------------------------- Alg. 2
def _run_reconcile(ctx, base, numel, n_freeze, seed):
    words = [torch.from_numpy(oracle.pack_bits(b).view(np.int32)).cuda() for b in base]
    stats = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    tf.tf_reconcile_mask(ctx, numel, words, n_freeze, seed, stats=stats)
    got = [oracle.unpack_bits(w.cpu().numpy().view("<u4"), n) for w, n in zip(words, numel)]
    raw = [w.cpu().numpy().view("<u4") for w in words]
    return got, raw, stats.cpu().numpy()


@pytest.mark.parametrize("density", [0.0, 0.3, 0.7, 1.0])
def test_reconcile_matches_the_oracle_bit_for_bit(ctx, density):
    rs = np.random.default_rng(int(density * 10) + 40)
    numel = [1, 31, 32, 33, 4097, 32768, 32769, 100003, 5]           # word / block boundaries and ragged tails
    N = sum(numel)
    base = [(rs.random(n) < density).astype(np.uint8) for n in numel]
    c = int(sum(int(b.sum()) for b in base))
    for r in (0.0, 0.25, 0.5, 0.9, 1.0):
        nf = math.floor(r * N)
        seed = 0xC0FFEE ^ (nf * 7919)
        got, raw, stats = _run_reconcile(ctx, base, numel, nf, seed)
        ref, count = oracle.reconcile_mask(base, numel, nf, seed)
        for g, e in zip(got, ref):
            assert np.array_equal(g, e)
        assert stats[0] == count == c
        assert stats[1] == (0 if c == nf else 1 if c < nf else 2)
        assert sum(int(g.sum()) for g in got) == nf
        for w, n in zip(raw, numel):                                   # bits past the end of a tensor stay clear
            if n % 32:
                assert int(w[-1]) >> (n % 32) == 0
    got, _, stats = _run_reconcile(ctx, base, numel, c, 5)             # budget already met
    assert all(np.array_equal(g, b) for g, b in zip(got, base)) and stats[1] == 0


def test_reconcile_more_tensors_than_one_launch_holds(ctx):
    rs = np.random.default_rng(8)
    numel = [int(n) for n in rs.integers(1, 3000, size=70)]           # 70 tensors: three launches per pass
    base = [(rs.random(n) < 0.4).astype(np.uint8) for n in numel]
    N = sum(numel)
    for nf in (N // 5, (4 * N) // 5):
        got, _, stats = _run_reconcile(ctx, base, numel, nf, 123456789)
        ref, _ = oracle.reconcile_mask(base, numel, nf, 123456789)
        assert all(np.array_equal(g, e) for g, e in zip(got, ref))


def test_reconcile_threshold_is_the_largest_key_drawn(ctx):
    rs = np.random.default_rng(3)
    numel = [50000, 70001]
    base = [(rs.random(n) < 0.5).astype(np.uint8) for n in numel]
    flat = np.concatenate(base)
    c, N = int(flat.sum()), sum(numel)
    keys = oracle.perm32(np.arange(N), 77).astype(np.int64)
    got, _, stats = _run_reconcile(ctx, base, numel, c + 1234, 77)
    new = np.concatenate(got)
    added = np.flatnonzero((new == 1) & (flat == 0))
    assert added.size == 1234 and stats[2] == keys[added].max()
    got, _, stats = _run_reconcile(ctx, base, numel, c - 999, 77)
    new = np.concatenate(got)
    dropped = np.flatnonzero((new == 0) & (flat == 1))
    assert dropped.size == 999 and stats[2] == keys[dropped].max()
