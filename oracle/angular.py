"""The target that RACE Attention estimates: attention with the P-powered angular kernel (Section 3.2, the
sharpened angular similarity; Section 3.4 / appendix "Target kernel").  fp64, quadratic in N.

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: it serves the approximation-quality checks (Theorem 1's bias
term P/beta and variance term sqrt(log N / L)), never the product path.
"""
from __future__ import annotations

import numpy as np


def angular_kernel(Q: np.ndarray, K: np.ndarray, gamma: float) -> np.ndarray:
    """S[i, j] = (1 - arccos(<Q_i, K_j> / (|Q_i| |K_j|)) / pi) ** gamma, in [0, 1]."""
    qn = Q / np.linalg.norm(Q, axis=1, keepdims=True)
    kn = K / np.linalg.norm(K, axis=1, keepdims=True)
    return (1.0 - np.arccos(np.clip(qn @ kn.T, -1.0, 1.0)) / np.pi) ** gamma


def angular_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, gamma: float, causal: bool = False):
    """O = D^-1 (M o S) V with the kernel above and row sums D (M: all ones, or the inclusive lower triangle)."""
    S = angular_kernel(Q, K, gamma)
    if causal:
        S = np.tril(S)
    return (S @ V) / S.sum(axis=1, keepdims=True)


def rms_error(O_hat: np.ndarray, O: np.ndarray) -> float:
    """Per-token root-mean-square error of Theorem 1: sqrt(mean_i |O_hat_i - O_i|_2^2)."""
    return float(np.sqrt(((O_hat - O) ** 2).sum(axis=1).mean()))
