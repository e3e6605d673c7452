"""ctypes front end of the C streaming oracle (oracle/race_oracle_stream.c).  Test infrastructure."""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        common = [ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                  ctypes.c_double, ctypes.c_int]
        lib.race_oracle_forward.argtypes = common + [dp] * 6
        lib.race_oracle_forward.restype = ctypes.c_int
        lib.race_oracle_backward.argtypes = common + [dp] * 11
        lib.race_oracle_backward.restype = ctypes.c_int
        lib.race_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _c(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def threads() -> int:
    return int(_load().race_oracle_threads())


def forward(Q, K, V, W, beta, L, P, causal):
    """Q, K, V: (B, H, N, d); W: (H, L*P, d).  Returns O (B, H, N, d) and Den (B, H, N)."""
    Q, K, V, W = _c(Q), _c(K), _c(V), _c(W)
    B, H, N, d = Q.shape
    assert W.shape == (H, L * P, d)
    O = np.empty_like(Q)
    den = np.empty((B, H, N))
    rc = _load().race_oracle_forward(B, H, N, d, L, P, float(beta), int(bool(causal)),
                                     _p(Q), _p(K), _p(V), _p(W), _p(O), _p(den))
    if rc:
        raise MemoryError("race_oracle_forward")
    return O, den


def backward(Q, K, V, W, beta, L, P, causal, O, den, dO, with_beta: bool = False):
    """Returns dQ, dK, dV and, if with_beta, the cotangent of the temperature per (batch, head), shape (B, H)."""
    Q, K, V, W, O, den, dO = map(_c, (Q, K, V, W, O, den, dO))
    B, H, N, d = Q.shape
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    dbeta = np.zeros((B, H))
    rc = _load().race_oracle_backward(B, H, N, d, L, P, float(beta), int(bool(causal)),
                                      _p(Q), _p(K), _p(V), _p(W), _p(O), _p(den), _p(dO),
                                      _p(dQ), _p(dK), _p(dV), _p(dbeta))
    if rc:
        raise MemoryError("race_oracle_backward")
    return (dQ, dK, dV, dbeta) if with_beta else (dQ, dK, dV)
