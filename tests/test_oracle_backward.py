"""Pins for the oracle's backward pass (derived from Algorithms 1/2; the paper prints no gradient)."""
import numpy as np
import pytest

from oracle import race_oracle as ro
from oracle import stream


def _data(N=24, d=6, L=3, P=3, seed=0, scale=0.6):
    rng = np.random.default_rng(seed)
    Q, K = (rng.standard_normal((N, d)) * scale for _ in range(2))
    V, dO = (rng.standard_normal((N, d)) for _ in range(2))
    W = ro.expand_projection(1, L, P, d)
    return Q, K, V, dO, W


@pytest.mark.parametrize("causal", [False, True])
def test_gradients_match_central_finite_differences(causal):
    Q, K, V, dO, W = _data()
    L, P, beta = 3, 3, 2.0
    grads = dict(zip("QKV", ro.backward_quadratic(Q, K, V, W, beta, L, P, causal, dO)))
    for which in "QKV":
        g = grads[which]
        fd = np.empty_like(g)
        for i in range(g.shape[0]):
            for c in range(g.shape[1]):
                fd[i, c] = ro.finite_difference(Q, K, V, W, beta, L, P, causal, dO, which, (i, c))
        assert np.abs(fd - g).max() < 1e-6 * max(1.0, np.abs(g).max()), which


@pytest.mark.parametrize("causal", [False, True])
def test_streaming_backward_equals_quadratic_backward(causal):
    Q, K, V, dO, W = _data(N=37, d=9)
    L, P, beta = 3, 3, 3.0
    g1 = ro.backward_quadratic(Q, K, V, W, beta, L, P, causal, dO)
    g2 = ro.backward_streaming(Q, K, V, W, beta, L, P, causal, dO)
    O, den = stream.forward(Q[None, None], K[None, None], V[None, None], W[None], beta, L, P, causal)
    g3 = stream.backward(Q[None, None], K[None, None], V[None, None], W[None], beta, L, P, causal,
                         O, den, dO[None, None])
    for a, b, c in zip(g1, g2, g3):
        scale = np.abs(a).max()
        assert np.abs(a - b).max() < 1e-11 * scale
        assert np.abs(a - c[0, 0]).max() < 1e-11 * scale


def test_c_oracle_many_heads_and_thread_independence():
    rng = np.random.default_rng(4)
    B, H, N, d, L, P, beta = 2, 3, 29, 8, 2, 2, 1.5
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    Ws = [ro.expand_projection(s, L, P, d) for s in range(H)]
    for causal in (False, True):
        O, den = stream.forward(Q, K, V, np.stack(Ws), beta, L, P, causal)
        got = stream.backward(Q, K, V, np.stack(Ws), beta, L, P, causal, O, den, dO)
        ref = ro.backward(Q, K, V, Ws, beta, L, P, causal, dO)
        for a, b in zip(ref, got):
            assert np.abs(a - b).max() < 1e-11 * np.abs(a).max()


@pytest.mark.parametrize("causal", [False, True])
def test_backward_invariants(causal):
    Q, K, V, dO, W = _data(N=31, d=7)
    L, P, beta = 3, 3, 2.0
    dQ, dK, dV = ro.backward_streaming(Q, K, V, W, beta, L, P, causal, dO)
    # rows of the attention matrix sum to one: total value gradient = total upstream gradient
    assert np.allclose(dV.sum(axis=0), dO.sum(axis=0), atol=1e-12)
    # a constant shift of V moves O by the same constant and leaves the weights alone
    dQ2, dK2, dV2 = ro.backward_streaming(Q, K, V + 3.0, W, beta, L, P, causal, dO)
    assert np.allclose(dQ, dQ2, atol=1e-11) and np.allclose(dK, dK2, atol=1e-11) and np.allclose(dV, dV2, atol=1e-13)
    if causal:
        # key/value j is never read by a query before it
        dO2 = dO.copy()
        dO2[:15] = 0.0
        _, dK3, dV3 = ro.backward_streaming(Q, K, V, W, beta, L, P, True, dO2)
        dO3 = dO - dO2
        _, dK4, dV4 = ro.backward_streaming(Q, K, V, W, beta, L, P, True, dO3)
        assert np.abs(dK4[15:]).max() == 0 and np.abs(dV4[15:]).max() == 0
        assert np.allclose(dK3 + dK4, dK, atol=1e-12)           # linear in dO


def test_a_planted_mistake_is_caught():
    # the finite-difference pin is sharp enough to see a dropped term: omit the normaliser cotangent
    Q, K, V, dO, W = _data(N=10, d=4)
    L, P, beta = 3, 3, 2.0
    good = ro.backward_quadratic(Q, K, V, W, beta, L, P, True, dO)[0]
    pq, pk = ro.soft_hash(Q, W, beta, L, P), ro.soft_hash(K, W, beta, L, P)
    S = np.tril(np.einsum("ilr,jlr->ij", pq, pk) / L)
    den = S.sum(axis=1)
    dS_wrong = np.tril(dO @ V.T) / den[:, None]                  # missing -(dO.O)/den
    bad = ro._soft_hash_vjp(Q, W, beta, L, P, np.einsum("ij,jlr->ilr", dS_wrong, pk) / L)
    fd = ro.finite_difference(Q, K, V, W, beta, L, P, True, dO, "Q", (3, 1))
    assert abs(fd - good[3, 1]) < 1e-7 and abs(fd - bad[3, 1]) > 1e-4


# ---------------------------------------------------------------- cotangent of the temperature beta
@pytest.mark.parametrize("causal", [False, True])
def test_beta_gradient_matches_central_differences(causal):
    rng = np.random.default_rng(11)
    N, d, L, P, beta = 9, 6, 3, 3, 1.7
    Q, K, V, dO = (rng.standard_normal((N, d)) * 0.6 for _ in range(4))
    W = rng.standard_normal((L * P, d))
    *_, db = ro.backward_quadratic(Q, K, V, W, beta, L, P, causal, dO, with_beta=True)
    fd = ro.finite_difference_beta(Q, K, V, W, beta, L, P, causal, dO)
    assert abs(db - fd) <= 1e-7 * max(1.0, abs(fd))
    *_, db_s = ro.backward_streaming(Q, K, V, W, beta, L, P, causal, dO, with_beta=True)
    assert abs(db_s - db) <= 1e-12 * max(1.0, abs(db))


def test_beta_gradient_by_hand_for_one_hyperplane():
    # P = 1, L = 1: phi = (sigma(-2 beta u), sigma(2 beta u)); with two tokens, non-causal, everything is explicit
    rng = np.random.default_rng(5)
    d, beta = 3, 0.9
    Q, K, V, dO = (rng.standard_normal((2, d)) for _ in range(4))
    W = rng.standard_normal((1, d))
    sig = lambda t: 1.0 / (1.0 + np.exp(-t))
    def loss(b):
        uq, uk = np.tanh(Q @ W[0]), np.tanh(K @ W[0])
        pq = np.stack([sig(-2 * b * uq), sig(2 * b * uq)], axis=1)
        pk = np.stack([sig(-2 * b * uk), sig(2 * b * uk)], axis=1)
        S = pq @ pk.T
        O = (S / S.sum(axis=1, keepdims=True)) @ V
        return float((dO * O).sum())
    h = 1e-6
    fd = (loss(beta + h) - loss(beta - h)) / (2 * h)
    *_, db = ro.backward_quadratic(Q, K, V, W, beta, 1, 1, False, dO, with_beta=True)
    assert abs(db - fd) <= 1e-7 * max(1.0, abs(fd))


def test_beta_gradient_c_oracle_matches_numpy_and_sums_over_heads():
    from oracle import stream as oracle_stream
    rng = np.random.default_rng(3)
    B, H, N, d, L, P, beta = 2, 2, 40, 8, 3, 3, 2.5
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) * 0.5 for _ in range(4))
    Ws = [rng.standard_normal((L * P, d)) for _ in range(H)]
    for causal in (False, True):
        O, den = ro.forward(Q, K, V, Ws, beta, L, P, causal)
        *_, db = ro.backward(Q, K, V, Ws, beta, L, P, causal, dO, with_beta=True)
        *_, dbc = oracle_stream.backward(Q, K, V, np.stack(Ws), beta, L, P, causal, O, den, dO, with_beta=True)
        assert db.shape == (B, H) and np.allclose(dbc, db, rtol=1e-10, atol=1e-12)
        # one beta for the whole layer: the loss is a sum over (batch, head), so is its derivative
        def loss(b):
            o, _ = ro.forward(Q, K, V, Ws, b, L, P, causal)
            return float((dO * o).sum())
        h = 1e-6
        fd = (loss(beta + h) - loss(beta - h)) / (2 * h)
        assert abs(db.sum() - fd) <= 1e-6 * max(1.0, abs(fd))


def test_beta_l1_scale_is_the_l1_norm_of_terms_that_sum_to_the_finite_difference():
    # the tolerance scale of the d(beta) comparisons: its terms, summed with their signs, must be the derivative itself
    # (central differences in beta, independent of the backward code); flipping or scaling dO leaves or scales the norm
    rng = np.random.default_rng(2)
    N, d, L, P, beta = 12, 5, 2, 3, 3.0
    Q, K, V, dO = (rng.standard_normal((N, d)) for _ in range(4))
    W = rng.standard_normal((L * P, d))
    for causal in (False, True):
        tq, tk = ro.beta_cotangent_terms(Q, K, V, W, beta, L, P, causal, dO)
        assert tq.shape == (N, L, P) and tk.shape == (N, L, P)
        fd = ro.finite_difference_beta(Q, K, V, W, beta, L, P, causal, dO)
        assert abs(tq.sum() + tk.sum() - fd) <= 1e-6 * max(1.0, abs(fd))
        *_, db = ro.backward_quadratic(Q, K, V, W, beta, L, P, causal, dO, with_beta=True)
        l1 = ro.beta_cotangent_l1(Q, K, V, W, beta, L, P, causal, dO)
        assert abs(l1 - (np.abs(tq).sum() + np.abs(tk).sum())) <= 1e-12 * l1
        assert l1 >= abs(db) and l1 > 0
        assert abs(ro.beta_cotangent_l1(Q, K, V, W, beta, L, P, causal, -dO) - l1) <= 1e-12 * l1
        assert abs(ro.beta_cotangent_l1(Q, K, V, W, beta, L, P, causal, 3.0 * dO) - 3.0 * l1) <= 1e-12 * l1
    # one token (causal): O = V whatever beta is, every term vanishes
    tq, tk = ro.beta_cotangent_terms(Q[:1], K[:1], V[:1], W, beta, L, P, True, dO[:1])
    assert np.abs(tq).max() <= 1e-15 and np.abs(tk).max() <= 1e-15
