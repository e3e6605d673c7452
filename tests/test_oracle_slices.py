"""The C streaming oracle run slice by slice (carried bucket statistics) against the same oracle run whole: the
scans perform the same additions in the same order, so the results must be equal bit for bit.  This is what lets the
GPU parity tests walk a multi-million-token sequence in bounded host memory.  The whole-sequence form is itself pinned
to the N x N definition and to finite differences in test_oracle_forward.py / test_oracle_backward.py."""
import numpy as np
import pytest

from oracle import race_oracle as ro
from oracle import stream as oracle_stream


def _inputs(B, H, N, d, L, P, seed):
    rng = np.random.default_rng(seed)
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    Q /= np.linalg.norm(Q, axis=-1, keepdims=True)
    K /= np.linalg.norm(K, axis=-1, keepdims=True)
    W = np.stack([ro.expand_projection(100 + h, L, P, d) for h in range(H)])
    return Q, K, V, dO, W


@pytest.mark.parametrize("cuts", [[0, 97, 97, 200, 333], [0, 1, 2, 333], [0, 333]])
def test_sliced_runs_equal_the_whole_run_bit_for_bit(cuts):
    B, H, N, d, L, P, beta = 2, 2, 333, 16, 3, 3, 4.0
    Q, K, V, dO, W = _inputs(B, H, N, d, L, P, 7)
    O, den = oracle_stream.forward(Q, K, V, W, beta, L, P, True)
    dQ, dK, dV = oracle_stream.backward(Q, K, V, W, beta, L, P, True, O, den, dO)

    sl = [slice(a, b) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    cut = lambda T, s: np.ascontiguousarray(T[:, :, s])
    # left to right: the forward pass and the query pass of the backward pass, each carrying its own statistics
    st_f, st_q = oracle_stream.new_state(B, H, L, P, d), oracle_stream.new_state(B, H, L, P, d)
    O2, den2, dQ2 = np.empty_like(O), np.empty_like(den), np.empty_like(dQ)
    for s in sl:
        O2[:, :, s], den2[:, :, s] = oracle_stream.forward_slice(cut(Q, s), cut(K, s), cut(V, s), W, beta, L, P, st_f)
        dQ2[:, :, s] = oracle_stream.backward_slice(cut(Q, s), cut(K, s), cut(V, s), W, beta, L, P, cut(O2, s),
                                                    np.ascontiguousarray(den2[:, :, s]), cut(dO, s), prefix_state=st_q)[0]
    assert np.array_equal(O2, O) and np.array_equal(den2, den) and np.array_equal(dQ2, dQ)
    # both passes leave the statistics of all keys and values behind
    assert np.array_equal(st_f, st_q)
    for b in range(B):
        for h in range(H):
            A, Bsum = ro.bucket_statistics(K[b, h], V[b, h], W[h], beta, L, P)
            assert np.allclose(st_f[b, h, :, :, d], A, rtol=1e-12, atol=1e-14)
            assert np.allclose(st_f[b, h, :, :, :d], Bsum, rtol=1e-12, atol=1e-13)
    # right to left: the key/value pass carrying the statistics of the read-out cotangents
    st_k = oracle_stream.new_state(B, H, L, P, d)
    dK2, dV2 = np.empty_like(dK), np.empty_like(dV)
    for s in reversed(sl):
        _, dK2[:, :, s], dV2[:, :, s] = oracle_stream.backward_slice(cut(Q, s), cut(K, s), cut(V, s), W, beta, L, P,
                                                                     cut(O, s), np.ascontiguousarray(den[:, :, s]),
                                                                     cut(dO, s), suffix_state=st_k)
    assert np.array_equal(dK2, dK) and np.array_equal(dV2, dV)


def test_a_tail_window_gives_the_key_and_value_gradients_of_its_tokens():
    """dK_j and dV_j of a causal layer depend on the tokens i >= j only once O and Den are given (the suffix statistics
    of the read-out cotangents): the key/value pass on the last n0 tokens alone, from an empty suffix, reproduces
    them.  (The full-size GPU tests use exactly this to check dK and dV at the far end of a 12 M-token sequence.)"""
    B, H, N, d, L, P, beta = 1, 2, 200, 16, 4, 3, 6.0
    Q, K, V, dO, W = _inputs(B, H, N, d, L, P, 11)
    O, den = oracle_stream.forward(Q, K, V, W, beta, L, P, True)
    _, dK, dV = oracle_stream.backward(Q, K, V, W, beta, L, P, True, O, den, dO)
    s = slice(N - 70, N)
    cut = lambda T: np.ascontiguousarray(T[:, :, s])
    _, dKw, dVw = oracle_stream.backward_slice(cut(Q), cut(K), cut(V), W, beta, L, P, cut(O), cut(den), cut(dO),
                                               suffix_state=oracle_stream.new_state(B, H, L, P, d))
    assert np.array_equal(dKw, dK[:, :, s]) and np.array_equal(dVw, dV[:, :, s])
    # and it is a property of the definition, not of this implementation: the N x N form agrees
    for h in range(H):
        _, rK, rV = ro.backward_quadratic(Q[0, h], K[0, h], V[0, h], W[h], beta, L, P, True, dO[0, h])
        assert np.allclose(dKw[0, h], rK[s], rtol=1e-9, atol=1e-12) and np.allclose(dVw[0, h], rV[s], rtol=1e-9, atol=1e-12)


def test_carried_statistics_are_for_the_causal_scan_only():
    B, H, N, d, L, P = 1, 1, 8, 8, 2, 2
    Q, K, V, dO, W = _inputs(B, H, N, d, L, P, 3)
    import ctypes
    lib = oracle_stream._load()
    st = oracle_stream.new_state(B, H, L, P, d)
    O, den = np.empty_like(Q), np.empty((B, H, N))
    p = oracle_stream._p
    assert lib.race_oracle_forward_carry(B, H, N, d, L, P, 4.0, 0, p(Q), p(K), p(V), p(W), p(st), p(O), p(den)) == 2
