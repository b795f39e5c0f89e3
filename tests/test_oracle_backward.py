"""Pins for the oracle's stage backward (Sec. 3.2.1 backward decomposition;
App. D.1 mask convention).  None of these re-types the oracle's loops: they
use finite differences of the forward bilinear form, numpy's matmul, adjoint
identities and special cases with known answers."""
import numpy as np
import pytest

import oracle


def _rand_layers(rs, shapes, T):
    W = [rs.standard_normal((k, n)) for k, n in shapes]
    X = [rs.standard_normal((T, k)) for k, n in shapes]
    dY = [rs.standard_normal((T, n)) for k, n in shapes]
    return W, X, dY


def _run(shapes, T, W, X, dY, mask, dW_init=None, accumulate=False):
    dX = [np.full((T, k), np.nan) for k, n in shapes]
    if dW_init is None:
        dW = [np.full((k, n), np.nan) for k, n in shapes]
    else:
        dW = [a.copy() for a in dW_init]
    oracle.stage_backward(shapes, T, W, X, dY, mask, dX, dW, accumulate=accumulate)
    return dX, dW


def test_finite_differences_of_bilinear_form():
    # l(X, W) = sum_l <dY_l, X_l W_l>;  dl/dX_l = dX_l, dl/dW_l = dW_l.
    rs = np.random.default_rng(1)
    shapes = [(4, 5), (3, 2)]
    T = 3
    W, X, dY = _rand_layers(rs, shapes, T)
    dX, dW = _run(shapes, T, W, X, dY, [0, 0])

    def loss(Xs, Ws):
        return sum(float(np.sum(dY[l] * (Xs[l] @ Ws[l]))) for l in range(len(shapes)))

    h = 1e-3  # central difference is exact for a bilinear form up to round-off
    for l, (k, n) in enumerate(shapes):
        for idx in np.ndindex(T, k):
            Xp = [a.copy() for a in X]; Xm = [a.copy() for a in X]
            Xp[l][idx] += h; Xm[l][idx] -= h
            fd = (loss(Xp, W) - loss(Xm, W)) / (2 * h)
            assert abs(fd - dX[l][idx]) < 1e-9 * max(1.0, abs(fd))
        for idx in np.ndindex(k, n):
            Wp = [a.copy() for a in W]; Wm = [a.copy() for a in W]
            Wp[l][idx] += h; Wm[l][idx] -= h
            fd = (loss(X, Wp) - loss(X, Wm)) / (2 * h)
            assert abs(fd - dW[l][idx]) < 1e-9 * max(1.0, abs(fd))


@pytest.mark.parametrize("T,shapes", [(7, [(5, 3), (3, 11)]), (33, [(17, 29), (64, 8), (1, 1)])])
def test_against_numpy_matmul(T, shapes):
    rs = np.random.default_rng(2)
    W, X, dY = _rand_layers(rs, shapes, T)
    dX, dW = _run(shapes, T, W, X, dY, [0] * len(shapes))
    for l in range(len(shapes)):
        np.testing.assert_allclose(dX[l], dY[l] @ W[l].T, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(dW[l], X[l].T @ dY[l], rtol=1e-12, atol=1e-12)


def test_adjoint_identities():
    # <dX, U> = <dY, U W>   and   <dW, V> = <X V, dY>
    rs = np.random.default_rng(3)
    shapes = [(13, 6), (6, 21)]
    T = 10
    W, X, dY = _rand_layers(rs, shapes, T)
    dX, dW = _run(shapes, T, W, X, dY, [0, 0])
    for l, (k, n) in enumerate(shapes):
        U = rs.standard_normal((T, k))
        V = rs.standard_normal((k, n))
        assert np.isclose(np.sum(dX[l] * U), np.sum(dY[l] * (U @ W[l])), rtol=1e-11)
        assert np.isclose(np.sum(dW[l] * V), np.sum((X[l] @ V) * dY[l]), rtol=1e-11)


def test_special_cases():
    rs = np.random.default_rng(4)
    # T = 1: dW is the outer product x^T dy; dX is W dy.
    k, n = 5, 4
    W = [rs.standard_normal((k, n))]
    x = rs.standard_normal((1, k)); dy = rs.standard_normal((1, n))
    dX, dW = _run([(k, n)], 1, W, [x], [dy], [0])
    for a in range(k):
        for b in range(n):
            assert dW[0][a, b] == x[0, a] * dy[0, b]
        assert np.isclose(dX[0][0, a], sum(W[0][a, b] * dy[0, b] for b in range(n)), rtol=1e-14)
    # W = I: dX = dY exactly.
    k = 6
    X = [rs.standard_normal((3, k))]; dY = [rs.standard_normal((3, k))]
    dX, _ = _run([(k, k)], 3, [np.eye(k)], X, dY, [0])
    assert np.array_equal(dX[0], dY[0])
    # one-hot dY at (t0, n0): dX[t0, :] = W[:, n0], other rows 0; dW[:, n0] = X[t0, :], others 0.
    k, n, T = 4, 7, 5
    W = [rs.standard_normal((k, n))]; X = [rs.standard_normal((T, k))]
    dY = [np.zeros((T, n))]; dY[0][2, 3] = 1.0
    dX, dW = _run([(k, n)], T, W, X, dY, [0])
    exp_dX = np.zeros((T, k)); exp_dX[2] = W[0][:, 3]
    exp_dW = np.zeros((k, n)); exp_dW[:, 3] = X[0][2]
    assert np.array_equal(dX[0], exp_dX)
    assert np.array_equal(dW[0], exp_dW)


def _canary(shape):
    # NaN payload pattern: any arithmetic on it or any rewrite with a computed value changes the bits
    a = np.empty(shape, dtype=np.float64)
    a.view(np.uint64)[...] = np.uint64(0x7FF8DEADBEEF0000) + np.arange(a.size, dtype=np.uint64).reshape(shape)
    return a


def test_freeze_mask_semantics():
    rs = np.random.default_rng(5)
    shapes = [(4, 3), (5, 2), (3, 3)]
    T = 6
    W, X, dY = _rand_layers(rs, shapes, T)
    can = [_canary(s) for s in shapes]
    # nothing frozen (r = 0): the full backward
    dX0, dW0 = _run(shapes, T, W, X, dY, [0, 0, 0], dW_init=can)
    for l in range(3):
        np.testing.assert_allclose(dW0[l], X[l].T @ dY[l], rtol=1e-12)
    # everything frozen (r = 1): every dW byte-identical, dX identical to r = 0
    dX1, dW1 = _run(shapes, T, W, X, dY, [1, 1, 1], dW_init=can)
    for l in range(3):
        assert dW1[l].tobytes() == can[l].tobytes()
        assert dX1[l].tobytes() == dX0[l].tobytes()
    # mixed: 1 = frozen (not the other way round)
    dX2, dW2 = _run(shapes, T, W, X, dY, [0, 1, 0], dW_init=can)
    assert dW2[1].tobytes() == can[1].tobytes()
    assert dW2[0].tobytes() == dW0[0].tobytes() and dW2[2].tobytes() == dW0[2].tobytes()
    assert all(dX2[l].tobytes() == dX0[l].tobytes() for l in range(3))
    # frozen dW may be absent altogether
    dX = [np.empty((T, k)) for k, n in shapes]
    oracle.stage_backward(shapes, T, W, X, dY, [1, 1, 1], dX, [None, None, None])
    assert all(dX[l].tobytes() == dX0[l].tobytes() for l in range(3))


def test_accumulate_sums_masked_microbatch_gradients():
    # sum_m U_m (.) g_m (App. D.1, update rule): a tensor frozen in microbatch m
    # contributes nothing from m; division by M is NOT done here.
    rs = np.random.default_rng(6)
    shapes = [(3, 4), (2, 5)]
    T, M = 4, 3
    W = [rs.standard_normal(s) for s in shapes]
    masks = [[0, 0], [1, 0], [0, 1]]
    acc = [np.zeros(s) for s in shapes]
    expect = [np.zeros(s) for s in shapes]
    for m in range(M):
        X = [rs.standard_normal((T, k)) for k, n in shapes]
        dY = [rs.standard_normal((T, n)) for k, n in shapes]
        dX = [np.empty((T, k)) for k, n in shapes]
        oracle.stage_backward(shapes, T, W, X, dY, masks[m], dX, acc, accumulate=True)
        for l in range(2):
            if not masks[m][l]:
                expect[l] += X[l].T @ dY[l]
    for l in range(2):
        np.testing.assert_allclose(acc[l], expect[l], rtol=1e-12, atol=1e-13)


def test_planted_transpose_would_be_caught():
    # sanity of the pins themselves: the transposed product differs from the right one
    rs = np.random.default_rng(7)
    k = n = 4; T = 4
    W = [rs.standard_normal((k, n))]; X = [rs.standard_normal((T, k))]; dY = [rs.standard_normal((T, n))]
    dX, dW = _run([(k, n)], T, W, X, dY, [0])
    assert not np.allclose(dX[0], dY[0] @ W[0])          # W, not W^T: wrong
    assert not np.allclose(dW[0], dY[0].T @ X[0])        # dY^T X: wrong


def test_sampled_elements_equal_the_full_oracle():
    # the one-by-one form used for outputs too large to compute in full
    rs = np.random.default_rng(8)
    k, n, T = 9, 13, 17
    W = [rs.standard_normal((k, n))]; X = [rs.standard_normal((T, k))]; dY = [rs.standard_normal((T, n))]
    dX, dW = _run([(k, n)], T, W, X, dY, [0])
    ts = rs.integers(0, T, 40); ks = rs.integers(0, k, 40); ns = rs.integers(0, n, 40)
    np.testing.assert_allclose(oracle.sample_dx(dY[0], W[0], ts, ks), dX[0][ts, ks], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.sample_dw(X[0], dY[0], ks, ns), dW[0][ks, ns], rtol=1e-13, atol=1e-14)
    # float32 inputs are up-cast exactly, not rounded
    got = oracle.sample_dx(dY[0].astype(np.float32), W[0].astype(np.float32), ts, ks)
    exp = (dY[0].astype(np.float32).astype(np.float64) @ W[0].astype(np.float32).astype(np.float64).T)[ts, ks]
    np.testing.assert_allclose(got, exp, rtol=1e-13, atol=1e-14)


def test_shared_input_gradient_is_the_product_with_the_concatenated_weights():
    """q, k, v (and gate, up) read the same activations: the gradient with respect to them is the
    sum of the members' products = dY_cat W_cat^T with the weights concatenated along the output
    features (Sec. 3.2.1: the activation-gradient component; the stage's linears as in a block)."""
    rng = np.random.default_rng(12)
    T, d, kv, ffn = 7, 6, 3, 10
    shapes = [(d, d), (d, kv), (d, kv), (d, d), (d, ffn), (d, ffn), (ffn, d)]
    groups = [0, 0, 0, -1, 1, 1, -1]
    W = [rng.standard_normal(s) for s in shapes]
    X = [rng.standard_normal((T, k)) for k, n in shapes]
    dY = [rng.standard_normal((T, n)) for k, n in shapes]
    dX = [np.zeros((T, k)) for k, n in shapes]
    dW = [np.zeros(s) for s in shapes]
    oracle.stage_backward_shared(shapes, T, W, X, dY, np.zeros(7, np.uint8), groups, dX, dW)
    qkv = np.concatenate(dY[0:3], axis=1) @ np.concatenate(W[0:3], axis=1).T
    gu = np.concatenate(dY[4:6], axis=1) @ np.concatenate(W[4:6], axis=1).T
    for l in (0, 1, 2):
        assert np.allclose(dX[l], qkv, atol=1e-12)
    for l in (4, 5):
        assert np.allclose(dX[l], gu, atol=1e-12)
    assert np.allclose(dX[3], dY[3] @ W[3].T, atol=1e-12) and np.allclose(dX[6], dY[6] @ W[6].T, atol=1e-12)
    for l in range(7):
        assert np.allclose(dW[l], X[l].T @ dY[l], atol=1e-12)           # weight gradients stay per layer
    # no groups: the plain backward
    dX2 = [np.zeros((T, k)) for k, n in shapes]
    oracle.stage_backward_shared(shapes, T, W, X, dY, np.zeros(7, np.uint8), None, dX2, [np.zeros(s) for s in shapes])
    assert all(np.allclose(a, g @ w.T, atol=1e-12) for a, g, w in zip(dX2, dY, W))
