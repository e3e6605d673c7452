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
        lib.race_oracle_forward_carry.argtypes = common + [dp] * 7
        lib.race_oracle_forward_carry.restype = ctypes.c_int
        lib.race_oracle_backward_carry.argtypes = common + [dp] * 9 + [ctypes.c_int, ctypes.c_int] + [dp] * 4
        lib.race_oracle_backward_carry.restype = ctypes.c_int
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


def new_state(B, H, L, P, d):
    """Zeroed carried statistics (B, H, L, R, d+1): per bucket row the d sums, then the mass."""
    return np.zeros((B, H, L, 1 << P, d + 1))


def forward_slice(Q, K, V, W, beta, L, P, state):
    """Causal forward over one slice of a longer sequence (Algorithm 2 continued): starts from `state` (updated in
    place to the statistics after the slice's last token).  Returns O and Den of the slice."""
    Q, K, V, W = _c(Q), _c(K), _c(V), _c(W)
    B, H, N, d = Q.shape
    assert state.shape == (B, H, L, 1 << P, d + 1) and state.dtype == np.float64 and state.flags.c_contiguous
    O = np.empty_like(Q)
    den = np.empty((B, H, N))
    rc = _load().race_oracle_forward_carry(B, H, N, d, L, P, float(beta), 1, _p(Q), _p(K), _p(V), _p(W), _p(state),
                                           _p(O), _p(den))
    if rc:
        raise MemoryError("race_oracle_forward_carry rc=%d" % rc)
    return O, den


def backward_slice(Q, K, V, W, beta, L, P, O, den, dO, prefix_state=None, suffix_state=None):
    """Causal backward over one slice.  prefix_state given: runs the query pass from it (the statistics of the keys
    and values before the slice; advanced in place) and returns dQ.  suffix_state given: runs the key/value pass
    from it (the statistics of the read-out cotangents after the slice; advanced in place) and returns dK, dV.
    Returns (dQ or None, dK or None, dV or None)."""
    Q, K, V, W, O, den, dO = map(_c, (Q, K, V, W, O, den, dO))
    B, H, N, d = Q.shape
    for st in (prefix_state, suffix_state):
        assert st is None or (st.shape == (B, H, L, 1 << P, d + 1) and st.dtype == np.float64 and st.flags.c_contiguous)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    dbeta = np.zeros((B, H))
    null = ctypes.POINTER(ctypes.c_double)()
    rc = _load().race_oracle_backward_carry(B, H, N, d, L, P, float(beta), 1, _p(Q), _p(K), _p(V), _p(W), _p(O), _p(den),
                                            _p(dO), _p(prefix_state) if prefix_state is not None else null,
                                            _p(suffix_state) if suffix_state is not None else null,
                                            int(prefix_state is not None), int(suffix_state is not None),
                                            _p(dQ), _p(dK), _p(dV), _p(dbeta))
    if rc:
        raise MemoryError("race_oracle_backward_carry rc=%d" % rc)
    return (dQ if prefix_state is not None else None, dK if suffix_state is not None else None,
            dV if suffix_state is not None else None)
