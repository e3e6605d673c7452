"""The oracle's RACE layer against the attention it estimates (the P-powered angular kernel), on synthetic
unit-norm queries and keys: the two terms of Theorem 1.  Statistical checks of trends, with wide margins;
they pin the scaling of W (unit-variance projections), the kernel exponent gamma = P and the normalisation."""
import math

import numpy as np

from oracle import angular
from oracle import race_oracle as ro


def _unit_rows(rng, n, d):
    x = rng.standard_normal((n, d))
    return x / np.linalg.norm(x, axis=1, keepdims=True)


def _clustered(seed, N, d, centres=8, spread=0.35):
    """Queries and keys around a few shared directions, so that attention rows are far from uniform."""
    rng = np.random.default_rng(seed)
    c = _unit_rows(rng, centres, d)
    def draw():
        x = c[rng.integers(0, centres, N)] + spread * rng.standard_normal((N, d)) / math.sqrt(d)
        return x / np.linalg.norm(x, axis=1, keepdims=True)
    return draw(), draw(), rng.standard_normal((N, d))


def test_angular_kernel_by_hand():
    q = np.array([[1.0, 0.0], [0.0, 2.0]])
    k = np.array([[1.0, 0.0], [1.0, 1.0], [-3.0, 0.0]])
    S = angular.angular_kernel(q, k, 3)
    assert np.allclose(S[0], [1.0, 0.75 ** 3, 0.0]) and np.allclose(S[1], [0.125, 0.75 ** 3, 0.125])
    V = np.array([[1.0], [2.0], [4.0]])
    O = angular.angular_attention(q, k, V, 3)
    assert np.allclose(O[0, 0], (1.0 + 2 * 0.75 ** 3) / (1 + 0.75 ** 3))
    assert np.allclose(angular.angular_attention(q[:1], k[:1], V[:1], 3, causal=True), [[1.0]])


def test_hard_race_converges_to_angular_attention_like_one_over_sqrt_L():
    # variance term of Theorem 1: the hard layer is unbiased for the kernel, its error falls like L^-1/2
    N, d, P = 192, 16, 4
    Q, K, V = _clustered(3, N, d)
    target = angular.angular_attention(Q, K, V, P)
    errs = {}
    for L in (8, 32, 128, 512):
        e = []
        for rep in range(3):
            W = ro.expand_projection(1000 * L + rep, L, P, d)
            e.append(angular.rms_error(ro.forward_hard(Q, K, V, W, L, P, False)[0], target))
        errs[L] = float(np.mean(e))
    print("hard RACE vs angular attention, rms error by L:", {k: round(v, 4) for k, v in errs.items()})
    assert errs[8] > errs[32] > errs[128] > errs[512]
    for a, b in ((8, 128), (32, 512)):
        assert 2.5 < errs[a] / errs[b] < 6.5            # sqrt(16) = 4
    assert errs[512] < 0.1 * np.sqrt((target ** 2).sum(axis=1).mean()) + 0.05


def test_soft_race_bias_falls_with_the_temperature():
    # bias term of Theorem 1: with many tables the remaining error is the softening, which shrinks as beta grows
    N, d, P, L = 160, 16, 4, 384
    Q, K, V = _clustered(4, N, d)
    target = angular.angular_attention(Q, K, V, P)
    W = ro.expand_projection(77, L, P, d)
    hard = angular.rms_error(ro.forward_hard(Q, K, V, W, L, P, False)[0], target)
    errs = {b: angular.rms_error(ro.forward_linear(Q, K, V, W, b, L, P)[0], target) for b in (0.5, 2.0, 8.0, 32.0)}
    print("soft RACE vs angular attention, rms error by beta:", {k: round(v, 4) for k, v in errs.items()}, "hard:", round(hard, 4))
    assert errs[0.5] > errs[2.0] > errs[8.0]
    assert errs[0.5] > 3 * errs[32.0]
    assert abs(errs[32.0] - hard) < 0.5 * hard + 0.02    # large beta: only the variance of the hard layer is left
    # causal variant against the causally masked target (the theorem covers the non-causal case only)
    tc = angular.angular_attention(Q, K, V, P, causal=True)
    ec = angular.rms_error(ro.forward_quadratic(Q, K, V, W, 32.0, L, P, True)[0][N // 2:], tc[N // 2:])
    assert ec < 3 * errs[32.0] + 0.05
