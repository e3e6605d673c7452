"""Pins for the oracle's optional unit-norm queries and keys (the setting of Theorem 1's proof: |Q_i| = |K_j| = 1):
closed forms of the map x -> x / |x| and of its Jacobian, invariances of the layer behind it, and central finite
differences of the composed layer."""
import numpy as np
import pytest

from oracle import race_oracle as ro


def _data(N=20, d=6, L=3, P=3, seed=3):
    rng = np.random.default_rng(seed)
    Q, K = (rng.standard_normal((N, d)) * rng.uniform(0.2, 5.0, (N, 1)) for _ in range(2))
    V, dO = (rng.standard_normal((N, d)) for _ in range(2))
    W = ro.expand_projection(1, L, P, d)
    return Q, K, V, dO, W


def test_rows_get_unit_length_and_keep_their_direction():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((50, 7)) * rng.uniform(1e-3, 1e3, (50, 1))
    U = ro.unit_rows(X)
    assert np.allclose(np.linalg.norm(U, axis=1), 1.0, rtol=0, atol=1e-14)
    assert np.allclose(U * np.linalg.norm(X, axis=1, keepdims=True), X, rtol=1e-14)
    # a textbook case: (3, 4) -> (0.6, 0.8)
    assert np.allclose(ro.unit_rows(np.array([[3.0, 4.0]])), [[0.6, 0.8]], rtol=0, atol=1e-16)


def test_zero_and_tiny_rows_are_divided_by_the_floor():
    X = np.array([[0.0, 0.0, 0.0], [3e-13, 0.0, 4e-13]])
    U = ro.unit_rows(X)
    assert np.array_equal(U[0], np.zeros(3))
    assert np.allclose(U[1], [0.3, 0.0, 0.4])
    g = np.array([[1.0, 2.0, 3.0], [1.0, 2.0, 3.0]])
    assert np.allclose(ro.unit_rows_vjp(X, g), g / ro.UNIT_EPS)


def test_jacobian_closed_forms():
    x = np.array([[3.0, 4.0, 0.0]])
    # a radial cotangent is annihilated, a tangential one is divided by the length
    assert np.allclose(ro.unit_rows_vjp(x, np.array([[6.0, 8.0, 0.0]])), 0.0, atol=1e-15)
    assert np.allclose(ro.unit_rows_vjp(x, np.array([[0.0, 0.0, 2.5]])), [[0.0, 0.0, 0.5]])
    assert np.allclose(ro.unit_rows_vjp(x, np.array([[-4.0, 3.0, 0.0]])), [[-0.8, 0.6, 0.0]])
    # full Jacobian against (I - xhat xhat^T) / |x| written out
    rng = np.random.default_rng(1)
    x = rng.standard_normal((1, 5))
    n = np.linalg.norm(x)
    J = (np.eye(5) - np.outer(x[0], x[0]) / n ** 2) / n
    for c in range(5):
        e = np.zeros((1, 5)); e[0, c] = 1.0
        assert np.allclose(ro.unit_rows_vjp(x, e)[0], J[c], atol=1e-15)      # J is symmetric


def test_vjp_matches_finite_differences_of_the_map():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((4, 5)) * 3.0
    G = rng.standard_normal((4, 5))
    got = ro.unit_rows_vjp(X, G)
    h = 1e-6
    for i in range(4):
        for c in range(5):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, c] += h; Xm[i, c] -= h
            fd = ((ro.unit_rows(Xp) - ro.unit_rows(Xm)) * G).sum() / (2 * h)
            assert abs(fd - got[i, c]) < 1e-8


@pytest.mark.parametrize("causal", [False, True])
def test_layer_behind_unit_rows_ignores_row_lengths(causal):
    Q, K, V, dO, W = _data()
    L, P, beta = 3, 3, 2.5
    O1, den1 = ro.forward_quadratic(ro.unit_rows(Q), ro.unit_rows(K), V, W, beta, L, P, causal)
    rng = np.random.default_rng(9)
    Q2, K2 = Q * rng.uniform(0.1, 10.0, (Q.shape[0], 1)), K * rng.uniform(0.1, 10.0, (K.shape[0], 1))
    O2, den2 = ro.forward_quadratic(ro.unit_rows(Q2), ro.unit_rows(K2), V, W, beta, L, P, causal)
    assert np.allclose(O1, O2, rtol=1e-12, atol=1e-13) and np.allclose(den1, den2, rtol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
def test_composed_gradients_match_finite_differences_and_are_tangential(causal):
    Q, K, V, dO, W = _data()
    L, P, beta = 3, 3, 2.5

    def loss(q, k):
        O, _ = ro.forward_quadratic(ro.unit_rows(q), ro.unit_rows(k), V, W, beta, L, P, causal)
        return float((O * dO).sum())

    dQh, dKh, _ = ro.backward_quadratic(ro.unit_rows(Q), ro.unit_rows(K), V, W, beta, L, P, causal, dO)
    dQ, dK = ro.unit_rows_vjp(Q, dQh), ro.unit_rows_vjp(K, dKh)
    # the output does not depend on a row's length: the gradient has no component along the row
    for X, dX in ((Q, dQ), (K, dK)):
        assert np.abs((X * dX).sum(axis=1)).max() < 1e-12 * np.abs(dX).max() * np.abs(X).max()
    h = 1e-6
    for i in range(0, Q.shape[0], 3):
        for c in range(Q.shape[1]):
            Xp, Xm = Q.copy(), Q.copy()
            Xp[i, c] += h; Xm[i, c] -= h
            assert abs((loss(Xp, K) - loss(Xm, K)) / (2 * h) - dQ[i, c]) < 2e-7 * max(1.0, np.abs(dQ).max())
            Xp, Xm = K.copy(), K.copy()
            Xp[i, c] += h; Xm[i, c] -= h
            assert abs((loss(Q, Xp) - loss(Q, Xm)) / (2 * h) - dK[i, c]) < 2e-7 * max(1.0, np.abs(dK).max())
