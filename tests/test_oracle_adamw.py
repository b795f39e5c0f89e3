"""Pins for the oracle's masked AdamW step and APF recurrences (App. D.1 mask
convention; Sec. 2.3 APF; Table exp_setup names AdamW).  Closed forms derived
by hand, invariants, and independent bf16 roundings."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

HP = dict(lr=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def _state(n):
    return np.zeros(n), np.zeros(n)


def test_first_step_closed_form():
    # zero state, t = 1: m_hat = g, v_hat = g^2  =>  p1 = p0 (1 - lr wd) - lr g / (|g| + eps)
    rs = np.random.default_rng(0)
    n = 257
    p0 = rs.standard_normal(n) * 0.02
    g = rs.standard_normal(n) * 1e-3
    g[:3] = [0.0, 1e-12, -1e-12]          # eps matters here
    p = p0.copy(); m, v = _state(n)
    oracle.masked_adamw(p, m, v, g, step=1, **HP)
    exp = p0 * (1 - HP["lr"] * HP["weight_decay"]) - HP["lr"] * g / (np.abs(g) + HP["eps"])
    np.testing.assert_allclose(p, exp, rtol=1e-13, atol=1e-18)
    assert p[0] == p0[0] * (1 - HP["lr"] * HP["weight_decay"])   # g = 0: pure decay
    np.testing.assert_allclose(m, (1 - HP["beta1"]) * g, rtol=1e-14)
    np.testing.assert_allclose(v, (1 - HP["beta2"]) * g * g, rtol=1e-14)


def test_constant_gradient_n_steps_geometric_closed_form():
    # constant g: m_hat_t = g and v_hat_t = g^2 for every t (bias correction exact),
    # so p_t = a p_{t-1} - c with a = 1 - lr wd, c = lr g/(|g|+eps).
    rs = np.random.default_rng(1)
    n, steps = 64, 12
    p0 = rs.standard_normal(n) * 0.02
    g = rs.standard_normal(n) * 1e-3
    p = p0.copy(); m, v = _state(n)
    for t in range(1, steps + 1):
        oracle.masked_adamw(p, m, v, g, step=t, **HP)
    a = 1 - HP["lr"] * HP["weight_decay"]
    c = HP["lr"] * g / (np.abs(g) + HP["eps"])
    exp = a ** steps * p0 - c * (1 - a ** steps) / (1 - a)
    np.testing.assert_allclose(p, exp, rtol=1e-10)
    np.testing.assert_allclose(m, (1 - HP["beta1"] ** steps) * g, rtol=1e-12)
    np.testing.assert_allclose(v, (1 - HP["beta2"] ** steps) * g * g, rtol=1e-12)


def test_alternating_gradient_first_moment_closed_form():
    # g_t = (-1)^t g, wd = 0: v_hat = g^2 always;
    # m_t = (1-b1) g (-1)^t (1 - (-b1)^t) / (1 + b1)
    n, steps = 16, 9
    rs = np.random.default_rng(2)
    g = np.abs(rs.standard_normal(n)) * 1e-3 + 1e-4
    hp = dict(HP, weight_decay=0.0)
    p = np.zeros(n); m, v = _state(n)
    exp = np.zeros(n)
    b1 = hp["beta1"]
    for t in range(1, steps + 1):
        oracle.masked_adamw(p, m, v, ((-1) ** t) * g, step=t, **hp)
        m_t = (1 - b1) * g * (-1) ** t * (1 - (-b1) ** t) / (1 + b1)
        np.testing.assert_allclose(m, m_t, rtol=1e-12)
        exp -= hp["lr"] * (m_t / (1 - b1 ** t)) / (g + hp["eps"])
    np.testing.assert_allclose(p, exp, rtol=1e-11)


def test_two_steps_by_hand_second_moment():
    p0, a, b = 0.03, 2e-3, -5e-4
    lr, b1, b2, eps, wd = HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"]
    p = np.array([p0]); m, v = _state(1)
    oracle.masked_adamw(p, m, v, np.array([a]), step=1, **HP)
    oracle.masked_adamw(p, m, v, np.array([b]), step=2, **HP)
    p1 = p0 * (1 - lr * wd) - lr * a / (abs(a) + eps)
    m2 = b1 * (1 - b1) * a + (1 - b1) * b
    v2 = b2 * (1 - b2) * a * a + (1 - b2) * b * b
    p2 = p1 * (1 - lr * wd) - lr * (m2 / (1 - b1 ** 2)) / ((v2 / (1 - b2 ** 2)) ** 0.5 + eps)
    assert np.isclose(p[0], p2, rtol=1e-13)
    assert np.isclose(m[0], m2, rtol=1e-14) and np.isclose(v[0], v2, rtol=1e-14)


def test_step_is_the_bias_correction_exponent():
    g = np.array([1e-3]); t = 7
    p = np.array([0.0]); m, v = _state(1)
    hp = dict(HP, weight_decay=0.0, eps=0.0)
    oracle.masked_adamw(p, m, v, g, step=t, **hp)
    mhat = (1 - hp["beta1"]) / (1 - hp["beta1"] ** t)
    vhat = (1 - hp["beta2"]) / (1 - hp["beta2"] ** t)
    assert np.isclose(p[0], -hp["lr"] * mhat / vhat ** 0.5, rtol=1e-13)
    with pytest.raises(ValueError):
        oracle.masked_adamw(p, m, v, g, step=0, **hp)


def test_sign_step_when_betas_zero():
    rs = np.random.default_rng(3)
    g = rs.standard_normal(32)
    hp = dict(lr=1e-2, beta1=0.0, beta2=0.0, eps=0.0, weight_decay=0.0)
    p = np.zeros(32); m = rs.standard_normal(32); v = np.abs(rs.standard_normal(32))
    oracle.masked_adamw(p, m, v, g, step=3, **hp)
    np.testing.assert_allclose(p, -1e-2 * np.sign(g), rtol=1e-14)


def test_grad_scale_is_applied_to_the_gradient():
    rs = np.random.default_rng(4)
    n = 50
    g = rs.standard_normal(n) * 1e-3
    p0 = rs.standard_normal(n) * 0.02
    pa, pb = p0.copy(), p0.copy()
    ma, va = _state(n); mb, vb = _state(n)
    oracle.masked_adamw(pa, ma, va, g, step=1, grad_scale=0.125, **HP)     # 1/M with M = 8
    oracle.masked_adamw(pb, mb, vb, g * 0.125, step=1, **HP)
    assert pa.tobytes() == pb.tobytes() and ma.tobytes() == mb.tobytes() and va.tobytes() == vb.tobytes()


def test_frozen_elements_are_untouched_everywhere():
    rs = np.random.default_rng(5)
    n = 300
    arrs = {k: rs.standard_normal(n) for k in "pmgEA"}
    arrs["v"] = np.abs(rs.standard_normal(n))
    lowp = rs.standard_normal(n)
    frozen = (rs.random(n) < 0.5).astype(np.uint8)
    before = {k: a.copy() for k, a in arrs.items()}; lowp0 = lowp.copy()
    oracle.masked_adamw(arrs["p"], arrs["m"], arrs["v"], arrs["g"], step=4, p_lowp=lowp,
                        elem_frozen=frozen, ema=arrs["E"], ema_abs=arrs["A"], ema_decay=0.99, **HP)
    f = frozen.astype(bool)
    for k in "pmvEA":
        assert arrs[k][f].tobytes() == before[k][f].tobytes()        # I = 1: no update
        assert not np.any(arrs[k][~f] == before[k][~f])              # I = 0: updated
    assert lowp[f].tobytes() == lowp0[f].tobytes()
    # the unfrozen part equals an unmasked run on those elements alone
    sub = {k: before[k][~f].copy() for k in "pmvgEA"}
    oracle.masked_adamw(sub["p"], sub["m"], sub["v"], sub["g"], step=4,
                        ema=sub["E"], ema_abs=sub["A"], ema_decay=0.99, **HP)
    for k in "pmvEA":
        assert arrs[k][~f].tobytes() == sub[k].tobytes()
    # all frozen (r = 1): bit-identical state
    allf = np.ones(n, dtype=np.uint8)
    snap = {k: a.copy() for k, a in arrs.items()}
    oracle.masked_adamw(arrs["p"], arrs["m"], arrs["v"], arrs["g"], step=5, elem_frozen=allf,
                        ema=arrs["E"], ema_abs=arrs["A"], ema_decay=0.99, **HP)
    for k in "pmvEA":
        assert arrs[k].tobytes() == snap[k].tobytes()


def test_bf16_rounding_against_two_other_implementations():
    # exact cases
    assert oracle.bf16_rne(1.0) == 1.0
    assert oracle.bf16_rne(1.0 + 2.0 ** -8) == 1.0                  # tie -> even mantissa
    assert oracle.bf16_rne(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6  # tie -> even mantissa
    assert oracle.bf16_rne(1.0 + 2.0 ** -8 + 2.0 ** -30) == 1.0 + 2.0 ** -7
    assert oracle.bf16_rne(-0.3) == -0.30078125
    assert oracle.bf16_rne(2.0 ** -133) == 2.0 ** -133              # smallest subnormal
    assert oracle.bf16_rne(2.0 ** -135) == 0.0
    assert oracle.bf16_rne(3.4e38) == float("inf")
    # random binary32 values: the bit-trick rounding of the input generator and torch's cast
    rs = np.random.default_rng(6)
    x = (rs.standard_normal(4000) * np.exp(rs.uniform(-20, 20, 4000))).astype(np.float32)
    mine = np.array([oracle.bf16_rne(float(t)) for t in x])
    bits = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x)).astype(np.float64)
    tor = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(mine, bits) and np.array_equal(mine, tor)
    # low-precision copy written by the optimizer is the rounding of the new p
    p = rs.standard_normal(100) * 0.02; m, v = _state(100); low = np.zeros(100)
    oracle.masked_adamw(p, m, v, rs.standard_normal(100) * 1e-3, step=1, p_lowp=low, **HP)
    assert np.array_equal(low, torch.from_numpy(p).to(torch.bfloat16).to(torch.float64).numpy())


def test_ema_closed_forms():
    a = 0.99
    c = -3e-4
    n = 40
    # constant Delta = c from zero: E_n = (1 - a^n) c, A_n = (1 - a^n)|c|, score 1
    E = np.zeros(3); A = np.zeros(3)
    for _ in range(n):
        oracle.stability_update(np.full(3, c), E, A, a)
    np.testing.assert_allclose(E, (1 - a ** n) * c, rtol=1e-12)
    np.testing.assert_allclose(A, (1 - a ** n) * abs(c), rtol=1e-12)
    np.testing.assert_allclose(oracle.elem_scores(E, A), 1.0, rtol=1e-12)
    # alternating Delta_k = (-1)^k c: |E_n| = (1-a)|c| |1-(-a)^n| / (1+a); score -> (1-a)/(1+a)
    E = np.zeros(1); A = np.zeros(1)
    n = 4001
    for k in range(1, n + 1):
        oracle.stability_update(np.array([(-1) ** k * c]), E, A, a)
    assert np.isclose(abs(E[0]), (1 - a) * abs(c) * abs(1 - (-a) ** n) / (1 + a), rtol=1e-9)
    assert np.isclose(A[0], (1 - a ** n) * abs(c), rtol=1e-10)
    assert np.isclose(oracle.elem_scores(E, A)[0], (1 - a) / (1 + a), rtol=1e-9)
    assert np.isclose((1 - a) / (1 + a), 0.0050251256, rtol=1e-8)


def test_fused_ema_tracks_the_applied_update():
    # betas = 0, wd = 0, eps = 0: u = -lr sign(g) every step -> constant Delta
    hp = dict(lr=1e-3, beta1=0.0, beta2=0.0, eps=0.0, weight_decay=0.0)
    g = np.array([2.0, -0.5])
    p = np.zeros(2); m, v = _state(2); E = np.zeros(2); A = np.zeros(2)
    n = 25
    for t in range(1, n + 1):
        oracle.masked_adamw(p, m, v, g, step=t, ema=E, ema_abs=A, ema_decay=0.9, **hp)
    u = -1e-3 * np.sign(g)
    np.testing.assert_allclose(E, (1 - 0.9 ** n) * u, rtol=1e-12)
    np.testing.assert_allclose(A, (1 - 0.9 ** n) * 1e-3, rtol=1e-12)
    # general case: Delta is p_new - p_old
    rs = np.random.default_rng(8)
    n = 64
    p = rs.standard_normal(n); p0 = p.copy(); m, v = _state(n)
    E = rs.standard_normal(n); A = np.abs(rs.standard_normal(n)); E0, A0 = E.copy(), A.copy()
    oracle.masked_adamw(p, m, v, rs.standard_normal(n), step=1, ema=E, ema_abs=A, ema_decay=0.99,
                        **dict(HP, lr=0.1))
    d = p - p0
    np.testing.assert_allclose(E, 0.99 * E0 + 0.01 * d, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(A, 0.99 * A0 + 0.01 * np.abs(d), rtol=1e-9, atol=1e-12)


def test_score_invariants_and_sums():
    rs = np.random.default_rng(9)
    n = 1000
    E = np.zeros(n); A = np.zeros(n)
    for _ in range(30):
        oracle.stability_update(rs.standard_normal(n), E, A, 0.95)
    s = oracle.elem_scores(E, A)
    assert np.all(s >= 0) and np.all(s <= 1 + 1e-15)          # triangle inequality
    se, sa = oracle.score_sums(E, A)
    assert np.isclose(se, np.abs(E).sum(), rtol=1e-13) and np.isclose(sa, A.sum(), rtol=1e-13)
    assert 0 <= oracle.tensor_score(se, sa) <= 1
    assert oracle.tensor_score(0.0, 0.0) == 1.0               # never updated: not evidence of stability
    assert oracle.elem_scores(np.zeros(2), np.zeros(2)).tolist() == [1.0, 1.0]
    # frozen elements keep E, A in the standalone form too
    fz = (rs.random(n) < 0.3).astype(np.uint8)
    E1, A1 = E.copy(), A.copy()
    oracle.stability_update(rs.standard_normal(n), E1, A1, 0.95, elem_frozen=fz)
    f = fz.astype(bool)
    assert E1[f].tobytes() == E[f].tobytes() and A1[f].tobytes() == A[f].tobytes()
    assert not np.any(E1[~f] == E[~f])


def test_selection_brute_force():
    rs = np.random.default_rng(10)
    for L in range(1, 7):
        for trial in range(6):
            sc = rs.integers(0, 3, size=L).astype(float) if trial % 2 else rs.random(L)
            prev = np.zeros(L, dtype=np.uint8)
            for n in range(L + 1):
                mask = oracle.select_lowest(sc, n)
                assert mask.sum() == n
                fz = [(sc[i], i) for i in range(L) if mask[i]]
                un = [(sc[i], i) for i in range(L) if not mask[i]]
                assert all(a < b for a, b in itertools.product(fz, un))   # unique answer
                assert np.all(mask >= prev)                               # nested in n
                prev = mask
    with pytest.raises(ValueError):
        oracle.select_lowest([0.1, 0.2], 3)


def test_frozen_count_rule():
    assert [oracle.n_frozen(r, 14) for r in (0.0, 0.5, 1.0)] == [0, 7, 14]
    assert [oracle.n_frozen(r, 28) for r in (0, .25, .5, .75, .9)] == [0, 7, 14, 21, 26]
    assert [oracle.n_frozen(r, 56) for r in (0, .5, .9)] == [0, 28, 51]
    assert [oracle.n_frozen(r, 56) for r in (.2, .4, .6, .8)] == [12, 23, 34, 45]
    assert [wl.n_frozen_tensors(r, 56) for r in (.2, .4, .6, .8)] == [12, 23, 34, 45]
    assert oracle.n_frozen(0.1 * 3, 10) == 3          # 0.30000000000000004 * 10 must not give 4
