"""Pins for the oracle's soft-LSH assignment and forward pass.

The paper prints no worked numerical example, so every pin is an identity, a closed form, a
limiting case that reduces to a textbook routine, or brute force on tiny inputs.
"""
import math

import numpy as np
import pytest

from oracle import race_oracle as ro
from oracle import stream


def _data(N=40, d=12, L=3, P=3, seed=0, wseed=1):
    rng = np.random.default_rng(seed)
    Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
    W = ro.expand_projection(wseed, L, P, d)
    return Q, K, V, W


# ---------------------------------------------------------------- soft-LSH assignment
def test_corner_bit_order():
    v = ro.corners(3)
    assert v.shape == (8, 3)
    assert list(v[0]) == [-1, -1, -1] and list(v[1]) == [1, -1, -1] and list(v[6]) == [-1, 1, 1]


@pytest.mark.parametrize("P", [1, 2, 4, 6])
def test_phi_is_probability_and_factorises(P):
    # proof of the bias lemma: the corner softmax factorises over the P coordinates,
    # phi_r = prod_t sigmoid(2 beta v_{r,t} u_t)
    L, d, beta = 2, 10, 1.7
    rng = np.random.default_rng(P)
    X = rng.standard_normal((25, d)) * 0.4
    W = ro.expand_projection(3, L, P, d)
    phi = ro.soft_hash(X, W, beta, L, P)
    assert phi.shape == (25, L, 1 << P)
    assert np.all(phi > 0) and np.allclose(phi.sum(axis=2), 1.0, atol=1e-14)
    u = np.tanh((X @ W.T).reshape(25, L, P))
    v = ro.corners(P)
    closed = np.prod(1.0 / (1.0 + np.exp(-2 * beta * u[:, :, None, :] * v[None, None])), axis=3)
    assert np.allclose(phi, closed, rtol=1e-13, atol=1e-15)
    # the arg-max corner is the sign pattern of the projection = the hard hash code
    assert np.array_equal(phi.argmax(axis=2), ro.hard_codes(X, W, L, P))


def test_phi_single_hyperplane_by_hand():
    W = np.array([[0.5, -1.0, 2.0]])
    x = np.array([[1.0, 2.0, 0.25]])            # z = 0.5 - 2 + 0.5 = -1
    beta = 0.75
    phi = ro.soft_hash(x, W, beta, 1, 1)[0, 0]
    u = math.tanh(-1.0)
    sig = 1 / (1 + math.exp(-2 * beta * u))
    assert np.allclose(phi, [1 - sig, sig], atol=1e-15)
    assert ro.hard_codes(x, W, 1, 1)[0, 0] == 0


def test_kernel_is_product_of_per_bit_agreements():
    # inner product of two Kronecker-factorised assignments = product of 2-point inner products
    Q, K, _, W = _data()
    L, P, beta = 3, 3, 2.5
    S = ro.kernel_matrix(Q, K, W, beta, L, P)
    pq = 1 / (1 + np.exp(-2 * beta * np.tanh(Q @ W.T)))      # (N, L*P): mass on the +1 side
    pk = 1 / (1 + np.exp(-2 * beta * np.tanh(K @ W.T)))
    agree = pq[:, None, :] * pk[None, :, :] + (1 - pq[:, None, :]) * (1 - pk[None, :, :])
    brute = agree.reshape(len(Q), len(K), L, P).prod(axis=3).mean(axis=2)
    assert np.allclose(S, brute, rtol=1e-12, atol=1e-15)


# ---------------------------------------------------------------- forward identities
@pytest.mark.parametrize("causal", [False, True])
def test_linear_time_forms_equal_the_definition(causal):
    Q, K, V, W = _data(N=53)
    L, P, beta = 3, 3, 3.0
    Oq, dq = ro.forward_quadratic(Q, K, V, W, beta, L, P, causal)
    Ol, dl = (ro.forward_streaming if causal else ro.forward_linear)(Q, K, V, W, beta, L, P)
    Oc, dc = stream.forward(Q[None, None], K[None, None], V[None, None], W[None], beta, L, P, causal)
    for O, dn in ((Ol, dl), (Oc[0, 0], dc[0, 0])):
        assert np.abs(O - Oq).max() < 1e-12 * np.abs(Oq).max()
        assert np.abs(dn - dq).max() < 1e-12 * np.abs(dq).max()


def test_causal_is_inclusive_mask_by_brute_force():
    # written out with Python loops, independent of tril and of the streaming order
    Q, K, V, W = _data(N=9, d=5, L=2, P=2)
    L, P, beta = 2, 2, 1.3
    pq, pk = ro.soft_hash(Q, W, beta, L, P), ro.soft_hash(K, W, beta, L, P)
    O, den = ro.forward_streaming(Q, K, V, W, beta, L, P)
    for i in range(9):
        num, dn = np.zeros(5), 0.0
        for j in range(i + 1):
            w = sum(float(pq[i, l] @ pk[j, l]) for l in range(L)) / L
            num += w * V[j]
            dn += w
        assert np.allclose(O[i], num / dn, atol=1e-14) and abs(den[i] - dn) < 1e-14


@pytest.mark.parametrize("causal", [False, True])
def test_attention_weights_are_a_convex_combination(causal):
    Q, K, V, W = _data()
    L, P, beta = 3, 3, 4.0
    S = ro.kernel_matrix(Q, K, W, beta, L, P)
    if causal:
        S = np.tril(S)
    A = S / S.sum(axis=1, keepdims=True)
    assert np.all(A >= 0) and np.allclose(A.sum(axis=1), 1, atol=1e-14)
    ones = np.full_like(V, 2.5)
    O, _ = ro.forward_quadratic(Q, K, ones, W, beta, L, P, causal)
    assert np.allclose(O, 2.5, atol=1e-13)
    c = np.linspace(-1, 1, V.shape[1])
    fwd = ro.forward_streaming if causal else ro.forward_linear
    O1, _ = fwd(Q, K, V, W, beta, L, P)
    O2, _ = fwd(Q, K, V + c, W, beta, L, P)
    assert np.allclose(O2, O1 + c, atol=1e-13)


def test_causal_boundary_rows():
    Q, K, V, W = _data()
    L, P, beta = 3, 3, 2.0
    Oc, dc = ro.forward_streaming(Q, K, V, W, beta, L, P)
    On, dn = ro.forward_linear(Q, K, V, W, beta, L, P)
    assert np.allclose(Oc[0], V[0], atol=1e-14)               # first query sees only its own key
    assert np.allclose(Oc[-1], On[-1], atol=1e-13)            # last query sees every key
    assert abs(dc[-1] - dn[-1]) < 1e-13
    assert np.all(dc > 0) and np.all(np.diff(dc[:1]) >= 0)


def test_causal_output_ignores_the_future():
    Q, K, V, W = _data()
    L, P, beta = 3, 3, 2.0
    O1, _ = ro.forward_streaming(Q, K, V, W, beta, L, P)
    K2, V2 = K.copy(), V.copy()
    K2[25:] += 3.0
    V2[25:] -= 7.0
    O2, _ = ro.forward_streaming(Q, K2, V2, W, beta, L, P)
    assert np.array_equal(O1[:25], O2[:25]) and not np.allclose(O1[25:], O2[25:])


@pytest.mark.parametrize("causal", [False, True])
def test_beta_to_zero_is_the_running_mean(causal):
    Q, K, V, W = _data()
    L, P = 3, 3
    fwd = ro.forward_streaming if causal else ro.forward_linear
    O, den = fwd(Q, K, V, W, 1e-9, L, P)
    N = len(V)
    if causal:
        ref = np.cumsum(V, axis=0) / np.arange(1, N + 1)[:, None]
        cnt = np.arange(1, N + 1)
    else:
        ref = np.broadcast_to(V.mean(axis=0), V.shape)
        cnt = np.full(N, N)
    assert np.allclose(O, ref, atol=1e-7)
    assert np.allclose(den, cnt / (1 << P), rtol=1e-7)       # uniform phi: each pair collides with mass 1/R


@pytest.mark.parametrize("causal", [False, True])
def test_beta_to_infinity_is_hard_race(causal):
    # Section 3.3: with the hard hash h(x) = sign(W x) a query reads the counters of its own bucket;
    # averaging L tables weights key j by the number of tables in which it collides with query i.
    rng = np.random.default_rng(5)
    N, d, L, P = 60, 8, 6, 2
    W = ro.expand_projection(11, L, P, d)
    def far_from_hyperplanes(n):
        out = []
        while len(out) < n:
            x = rng.standard_normal(d) * 2
            if np.abs(W @ x).min() > 0.5:
                out.append(x)
        return np.array(out)
    Q, K = far_from_hyperplanes(N), far_from_hyperplanes(N)
    V = rng.standard_normal((N, d))
    cq = [[sum(int(W[l * P + t] @ x >= 0) << t for t in range(P)) for l in range(L)] for x in Q]
    ck = [[sum(int(W[l * P + t] @ x >= 0) << t for t in range(P)) for l in range(L)] for x in K]
    assert np.array_equal(np.array(cq), ro.hard_codes(Q, W, L, P))
    O, den = (ro.forward_streaming if causal else ro.forward_linear)(Q, K, V, W, 60.0, L, P)
    checked = 0
    for i in range(N):
        js = range(i + 1) if causal else range(N)
        c = np.array([sum(cq[i][l] == ck[j][l] for l in range(L)) for j in js], dtype=float)
        if c.sum() == 0:
            continue                     # no collision in any table: the soft limit is 0/0
        ref = (c[:, None] * V[: len(c)]).sum(axis=0) / c.sum()
        assert np.allclose(O[i], ref, atol=1e-8)
        assert abs(den[i] - c.sum() / L) < 1e-8
        checked += 1
    assert checked > N // 2
    # bucket tap: with hard assignments A counts the keys per bucket, B sums their values
    A, B = ro.bucket_statistics(K, V, W, 60.0, L, P)
    for l in range(L):
        for r in range(1 << P):
            members = [j for j in range(N) if ck[j][l] == r]
            assert abs(A[l, r] - len(members)) < 1e-8
            assert np.allclose(B[l, r], V[members].sum(axis=0) if members else 0, atol=1e-8)


def test_noncausal_symmetries():
    Q, K, V, W = _data()
    L, P, beta = 3, 3, 2.0
    O, _ = ro.forward_linear(Q, K, V, W, beta, L, P)
    perm = np.random.default_rng(3).permutation(len(K))
    O2, _ = ro.forward_linear(Q, K[perm], V[perm], W, beta, L, P)
    assert np.allclose(O, O2, atol=1e-13)
    Wp = W.reshape(L, P, -1)[[2, 0, 1]].reshape(L * P, -1)      # permute the tables
    O3, _ = ro.forward_linear(Q, K, V, Wp, beta, L, P)
    assert np.allclose(O, O3, atol=1e-13)


def test_multi_head_wrappers_agree_with_c_oracle():
    rng = np.random.default_rng(8)
    B, H, N, d, L, P, beta = 2, 2, 33, 8, 2, 3, 2.0
    Q, K, V = (rng.standard_normal((B, H, N, d)) for _ in range(3))
    Ws = [ro.expand_projection(s, L, P, d) for s in (5, 6)]
    for causal in (False, True):
        O1, d1 = ro.forward(Q, K, V, Ws, beta, L, P, causal)
        O2, d2 = stream.forward(Q, K, V, np.stack(Ws), beta, L, P, causal)
        assert np.abs(O1 - O2).max() < 1e-13 and np.abs(d1 - d2).max() < 1e-13
    # heads use their own W
    assert not np.allclose(O1[:, 0], ro.forward(Q, K, V, Ws[::-1], beta, L, P, True)[0][:, 0])


# ---------------------------------------------------------------- the kernel RACE estimates
def test_collision_probability_matches_the_powered_angular_kernel():
    # Gaussian hyperplanes: P[h(q) = h(k)] = (1 - theta/pi)^P; this fixes "rows of W are N(0, I), unscaled"
    d, P, tables = 16, 3, 40000
    theta = 1.1
    q = np.zeros(d); q[0] = 1.0
    k = np.zeros(d); k[0], k[1] = math.cos(theta), math.sin(theta)
    W = ro.expand_projection(99, tables, P, d)
    cq = ro.hard_codes(q[None], W, tables, P)[0]
    ck = ro.hard_codes(k[None], W, tables, P)[0]
    p_hat = (cq == ck).mean()
    p = (1 - theta / math.pi) ** P
    assert abs(p_hat - p) < 4 * math.sqrt(p * (1 - p) / tables)
    # z = <w, x> is N(0, 1) for unit x (no 1/sqrt(d) anywhere)
    z = (W @ q)
    assert abs(z.var() - 1) < 4 * math.sqrt(2 / z.size)
    # soft kernel: |E[phi(q).phi(k)] - (1 - theta/pi)^P| <= 4P/(sqrt(2 pi) beta) + 2P exp(-2 tanh(1) beta)
    beta = 12.0
    pq = ro.soft_hash(q[None], W, beta, tables, P)[0]
    pk = ro.soft_hash(k[None], W, beta, tables, P)[0]
    soft = (pq * pk).sum(axis=1)
    bound = 4 * P / (math.sqrt(2 * math.pi) * beta) + 2 * P * math.exp(-2 * math.tanh(1) * beta)
    assert abs(soft.mean() - p) < bound + 4 * soft.std() / math.sqrt(tables)
    # and the soft estimate approaches the hard one as beta grows
    pq2 = ro.soft_hash(q[None], W, 200.0, tables, P)[0]
    pk2 = ro.soft_hash(k[None], W, 200.0, tables, P)[0]
    assert abs((pq2 * pk2).sum(axis=1).mean() - p_hat) < 0.01


def test_decode_steps_reproduce_the_causal_forward_and_the_state_is_the_bucket_statistics():
    rng = np.random.default_rng(21)
    N, d, L, P, beta = 17, 6, 3, 3, 2.0
    Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
    W = rng.standard_normal((L * P, d))
    O, den = ro.forward_streaming(Q, K, V, W, beta, L, P)
    state = np.zeros((L, 1 << P, d + 1))
    for t in range(N):
        o, dn = ro.decode_step(state, Q[t], K[t], V[t], W, beta, L, P)
        assert np.allclose(o, O[t], rtol=1e-12, atol=1e-14) and abs(dn - den[t]) <= 1e-12 * den[t]
    A, B = ro.bucket_statistics(K, V, W, beta, L, P)
    assert np.allclose(state[:, :, :d], B, rtol=1e-12, atol=1e-14) and np.allclose(state[:, :, d], A, rtol=1e-12)
    # resuming from the statistics of a prefix gives the same continuation
    n0 = 9
    A0, B0 = ro.bucket_statistics(K[:n0], V[:n0], W, beta, L, P)
    st = np.concatenate([B0, A0[:, :, None]], axis=2)
    for t in range(n0, N):
        o, _ = ro.decode_step(st, Q[t], K[t], V[t], W, beta, L, P)
        assert np.allclose(o, O[t], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
def test_hard_race_is_collision_count_attention_and_the_limit_of_the_soft_one(causal):
    # Section 3.3: with h(x) = sign(W x), key j gets weight (number of tables where it shares the query's bucket);
    # brute force over pairs, then the soft layer at a large temperature away from the hyperplanes.
    rng = np.random.default_rng(9)
    N, d, L, P = 70, 8, 5, 3
    W = ro.expand_projection(13, L, P, d)
    def far(n):
        out = []
        while len(out) < n:
            x = rng.standard_normal(d) * 2
            if np.abs(W @ x).min() > 0.5:
                out.append(x)
        return np.array(out)
    Q, K = far(N), far(N)
    V = rng.standard_normal((N, d))
    O, den = ro.forward_hard(Q, K, V, W, L, P, causal)
    cq, ck = ro.hard_codes(Q, W, L, P), ro.hard_codes(K, W, L, P)
    empty = 0
    for i in range(N):
        js = np.arange(i + 1) if causal else np.arange(N)
        c = (cq[i][None, :] == ck[js]).sum(axis=1).astype(float)       # collisions per key
        assert den[i] == c.sum() / L
        if c.sum() == 0:
            assert not O[i].any()
            empty += 1
        else:
            assert np.allclose(O[i], (c[:, None] * V[js]).sum(axis=0) / c.sum(), atol=1e-12)
    assert empty < N // 2
    Os, dens = ro.forward_quadratic(Q, K, V, W, 60.0, L, P, causal)
    keep = den > 0
    assert np.allclose(dens[keep], den[keep], atol=1e-8) and np.allclose(Os[keep], O[keep], atol=1e-7)
    # causal self-attention (Q = K): token i always meets itself in all L tables
    O2, den2 = ro.forward_hard(K, K, V, W, L, P, True)
    assert den2.min() >= 1.0 and np.allclose(O2[0], V[0])
