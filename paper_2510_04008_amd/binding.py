"""Thin ctypes binding of librace_attn.so: argument marshalling only.  Every step of the path runs in
the library's HIP kernels; torch is used for device memory and streams.  Names follow include/race_attn.h.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librace_attn.so")

RACE_OK, RACE_ERR_INVALID_ARG, RACE_ERR_UNSUPPORTED, RACE_ERR_WORKSPACE, RACE_ERR_HIP, RACE_ERR_NOT_READY = range(6)
RACE_F32, RACE_BF16 = 0, 1


class RaceAttnDesc(ctypes.Structure):
    """race_attn_desc_t"""
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int64), ("d", ctypes.c_int32),
                ("L", ctypes.c_int32), ("P", ctypes.c_int32), ("sharpening", ctypes.c_float),
                ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32), ("chunk", ctypes.c_int64),
                ("unit_qk", ctypes.c_int32)]


class RaceAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        text = lib().race_status_string(status).decode()
        detail = lib().race_attn_last_error().decode() if status in (RACE_ERR_HIP, RACE_ERR_NOT_READY, RACE_ERR_WORKSPACE) else ""
        super().__init__("%s: %s%s" % (where, text, (" (" + detail + ")") if detail else ""))


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the shared library; builds it first only if no built library is present."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        vp, u64p, fp, u8p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint64), ctypes.c_void_p, ctypes.c_void_p
        dp = ctypes.POINTER(RaceAttnDesc)
        L.race_attn_workspace_bytes.argtypes = [dp]
        L.race_attn_workspace_bytes.restype = ctypes.c_size_t
        L.race_attn_kernel_family.argtypes = [dp]
        L.race_attn_kernel_family.restype = ctypes.c_int
        L.race_attn_segment_tokens.argtypes = [dp]
        L.race_attn_segment_tokens.restype = ctypes.c_int64
        L.race_attn_fwd.argtypes = [dp, vp, vp, vp, u64p, vp, fp, vp, ctypes.c_size_t, vp]
        L.race_attn_fwd.restype = ctypes.c_int
        L.race_attn_fwd_static.argtypes = [dp, vp, vp, vp, u64p, vp, fp, vp]
        L.race_attn_fwd_static.restype = ctypes.c_int
        L.race_attn_bwd.argtypes = [dp, vp, vp, vp, vp, fp, vp, u64p, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.race_attn_bwd.restype = ctypes.c_int
        L.race_attn_bwd_beta.argtypes = [dp, vp, vp, vp, vp, fp, vp, u64p, vp, vp, vp, fp, vp, ctypes.c_size_t, vp]
        L.race_attn_bwd_beta.restype = ctypes.c_int
        L.race_attn_bwd_saved.argtypes = L.race_attn_bwd_beta.argtypes
        L.race_attn_bwd_saved.restype = ctypes.c_int
        L.race_attn_expand_projection.argtypes = [dp, u64p, ctypes.POINTER(ctypes.c_float)]
        L.race_attn_expand_projection.restype = ctypes.c_int
        L.race_attn_debug_hash.argtypes = [dp, vp, u64p, u8p, fp, vp, ctypes.c_size_t, vp]
        L.race_attn_debug_hash.restype = ctypes.c_int
        L.race_attn_debug_buckets.argtypes = [dp, vp, vp, u64p, fp, fp, vp, ctypes.c_size_t, vp]
        L.race_attn_debug_buckets.restype = ctypes.c_int
        L.race_attn_profile_enable.argtypes = [ctypes.c_int]
        L.race_attn_profile_enable.restype = None
        L.race_attn_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                             ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int)]
        L.race_attn_profile_read.restype = ctypes.c_int
        L.race_attn_calibration_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.race_attn_calibration_copy.restype = ctypes.c_int
        L.race_attn_state_bytes.argtypes = [dp]
        L.race_attn_state_bytes.restype = ctypes.c_size_t
        L.race_attn_state_init.argtypes = [dp, vp, vp, u64p, fp, vp, ctypes.c_size_t, vp]
        L.race_attn_state_init.restype = ctypes.c_int
        L.race_attn_step_workspace_bytes.argtypes = [dp]
        L.race_attn_step_workspace_bytes.restype = ctypes.c_size_t
        L.race_attn_step.argtypes = [dp, vp, vp, vp, u64p, fp, vp, fp, vp, ctypes.c_size_t, vp]
        L.race_attn_step.restype = ctypes.c_int
        L.race_attn_calibration_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, fp, vp]
        L.race_attn_calibration_mfma.restype = ctypes.c_int
        L.race_status_string.argtypes = [ctypes.c_int]
        L.race_status_string.restype = ctypes.c_char_p
        L.race_attn_last_error.argtypes = []
        L.race_attn_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def make_desc(B: int, H: int, N: int, d: int, L: int, P: int, sharpening: float, causal: bool,
              dtype: int, chunk: int = 0, unit_qk: bool = False) -> RaceAttnDesc:
    return RaceAttnDesc(B, H, N, d, L, P, float(sharpening), int(bool(causal)), int(dtype), int(chunk),
                        int(bool(unit_qk)))


def _seeds(seeds: Sequence[int]):
    arr = (ctypes.c_uint64 * len(seeds))(*[int(s) & 0xFFFFFFFFFFFFFFFF for s in seeds])
    return arr


def _torch():
    import torch
    return torch


def _elem_dtype(desc):
    torch = _torch()
    return torch.float32 if desc.dtype == RACE_F32 else torch.bfloat16


def _check_tensor(t, desc, name, shape=None, dtype=None):
    shape = shape or (desc.B, desc.H, desc.N, desc.d)
    dtype = dtype or _elem_dtype(desc)
    if not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != tuple(shape) or t.dtype != dtype:
        raise ValueError("%s must be a contiguous device tensor of shape %s and dtype %s" % (name, shape, dtype))


def _stream(stream) -> int:
    if stream is None:
        return _torch().cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _workspace(desc, workspace, device):
    torch = _torch()
    need = race_attn_workspace_bytes(desc)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel()


def race_attn_workspace_bytes(desc: RaceAttnDesc) -> int:
    return int(lib().race_attn_workspace_bytes(ctypes.byref(desc)))


def race_attn_kernel_family(desc: RaceAttnDesc) -> int:
    return int(lib().race_attn_kernel_family(ctypes.byref(desc)))


def race_attn_segment_tokens(desc: RaceAttnDesc) -> int:
    return int(lib().race_attn_segment_tokens(ctypes.byref(desc)))


def race_attn_expand_projection(desc: RaceAttnDesc, proj_seeds: Sequence[int]) -> np.ndarray:
    out = np.empty((desc.H, desc.L * desc.P, desc.d), dtype=np.float32)
    st = lib().race_attn_expand_projection(ctypes.byref(desc), _seeds(proj_seeds),
                                           out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_expand_projection")
    return out


def race_attn_fwd(desc: RaceAttnDesc, Q, K, V, proj_seeds: Sequence[int], O=None, den=None,
                  workspace=None, stream=None):
    torch = _torch()
    for t, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _check_tensor(t, desc, n)
    if O is None:
        O = torch.empty_like(V)
    if den is None:
        den = torch.empty((desc.B, desc.H, desc.N), dtype=torch.float32, device=V.device)
    _check_tensor(O, desc, "O")
    _check_tensor(den, desc, "den", (desc.B, desc.H, desc.N), torch.float32)
    workspace, nbytes = _workspace(desc, workspace, V.device)
    st = lib().race_attn_fwd(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _seeds(proj_seeds),
                             O.data_ptr(), den.data_ptr(), workspace.data_ptr(), nbytes, _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_fwd")
    return O, den


def race_attn_fwd_static(desc: RaceAttnDesc, Q, K, V, proj_seeds: Sequence[int], O, den, stream=None):
    """race_attn_fwd on the library's built-in scratch array; the caller passes every output (nothing is allocated)."""
    torch = _torch()
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O")):
        _check_tensor(t, desc, n)
    _check_tensor(den, desc, "den", (desc.B, desc.H, desc.N), torch.float32)
    st = lib().race_attn_fwd_static(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _seeds(proj_seeds),
                                    O.data_ptr(), den.data_ptr(), _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_fwd_static")
    return O, den


def race_attn_bwd(desc: RaceAttnDesc, Q, K, V, O, den, dO, proj_seeds: Sequence[int], dQ=None, dK=None, dV=None,
                  workspace=None, stream=None):
    torch = _torch()
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O"), (dO, "dO")):
        _check_tensor(t, desc, n)
    _check_tensor(den, desc, "den", (desc.B, desc.H, desc.N), torch.float32)
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    for t, n in ((dQ, "dQ"), (dK, "dK"), (dV, "dV")):
        _check_tensor(t, desc, n)
    workspace, nbytes = _workspace(desc, workspace, V.device)
    st = lib().race_attn_bwd(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                             den.data_ptr(), dO.data_ptr(), _seeds(proj_seeds), dQ.data_ptr(), dK.data_ptr(),
                             dV.data_ptr(), workspace.data_ptr(), nbytes, _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_bwd")
    return dQ, dK, dV


def race_attn_bwd_beta(desc: RaceAttnDesc, Q, K, V, O, den, dO, proj_seeds: Sequence[int], dQ=None, dK=None, dV=None,
                       dbeta=None, workspace=None, stream=None):
    """race_attn_bwd plus the cotangent of the temperature per (batch, head): returns dQ, dK, dV, dbeta (B, H)."""
    torch = _torch()
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O"), (dO, "dO")):
        _check_tensor(t, desc, n)
    _check_tensor(den, desc, "den", (desc.B, desc.H, desc.N), torch.float32)
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    for t, n in ((dQ, "dQ"), (dK, "dK"), (dV, "dV")):
        _check_tensor(t, desc, n)
    dbeta = torch.empty((desc.B, desc.H), dtype=torch.float32, device=V.device) if dbeta is None else dbeta
    _check_tensor(dbeta, desc, "dbeta", (desc.B, desc.H), torch.float32)
    workspace, nbytes = _workspace(desc, workspace, V.device)
    st = lib().race_attn_bwd_beta(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                  den.data_ptr(), dO.data_ptr(), _seeds(proj_seeds), dQ.data_ptr(), dK.data_ptr(),
                                  dV.data_ptr(), dbeta.data_ptr(), workspace.data_ptr(), nbytes, _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_bwd_beta")
    return dQ, dK, dV, dbeta


def race_attn_bwd_saved(desc: RaceAttnDesc, Q, K, V, O, den, dO, proj_seeds: Sequence[int], workspace, dQ=None, dK=None,
                        dV=None, dbeta=None, want_dbeta: bool = False, stream=None):
    """The backward pass on the workspace that race_attn_fwd of the same inputs left behind (required argument).
    Returns dQ, dK, dV and, if want_dbeta or dbeta is given, dbeta (B, H)."""
    torch = _torch()
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O"), (dO, "dO")):
        _check_tensor(t, desc, n)
    _check_tensor(den, desc, "den", (desc.B, desc.H, desc.N), torch.float32)
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    for t, n in ((dQ, "dQ"), (dK, "dK"), (dV, "dV")):
        _check_tensor(t, desc, n)
    if dbeta is None and want_dbeta:
        dbeta = torch.empty((desc.B, desc.H), dtype=torch.float32, device=V.device)
    if dbeta is not None:
        _check_tensor(dbeta, desc, "dbeta", (desc.B, desc.H), torch.float32)
    if workspace is None:
        raise ValueError("race_attn_bwd_saved needs the workspace the forward pass wrote")
    st = lib().race_attn_bwd_saved(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                   den.data_ptr(), dO.data_ptr(), _seeds(proj_seeds), dQ.data_ptr(), dK.data_ptr(),
                                   dV.data_ptr(), dbeta.data_ptr() if dbeta is not None else None,
                                   workspace.data_ptr(), workspace.numel(), _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_bwd_saved")
    return (dQ, dK, dV, dbeta) if dbeta is not None else (dQ, dK, dV)


def race_attn_debug_hash(desc: RaceAttnDesc, X, proj_seeds: Sequence[int], want_phi: bool = False,
                         workspace=None, stream=None):
    torch = _torch()
    _check_tensor(X, desc, "X")
    codes = torch.empty((desc.B, desc.H, desc.N, desc.L), dtype=torch.uint8, device=X.device)
    phi = torch.empty((desc.B, desc.H, desc.N, desc.L, 1 << desc.P), dtype=torch.float32,
                      device=X.device) if want_phi else None
    workspace, nbytes = _workspace(desc, workspace, X.device)
    st = lib().race_attn_debug_hash(ctypes.byref(desc), X.data_ptr(), _seeds(proj_seeds), codes.data_ptr(),
                                    phi.data_ptr() if want_phi else None, workspace.data_ptr(), nbytes,
                                    _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_debug_hash")
    return codes, phi


def race_attn_debug_buckets(desc: RaceAttnDesc, K, V, proj_seeds: Sequence[int], workspace=None, stream=None):
    torch = _torch()
    _check_tensor(K, desc, "K")
    _check_tensor(V, desc, "V")
    R = 1 << desc.P
    A = torch.empty((desc.B, desc.H, desc.L, R), dtype=torch.float32, device=K.device)
    Bsum = torch.empty((desc.B, desc.H, desc.L, R, desc.d), dtype=torch.float32, device=K.device)
    workspace, nbytes = _workspace(desc, workspace, K.device)
    st = lib().race_attn_debug_buckets(ctypes.byref(desc), K.data_ptr(), V.data_ptr(), _seeds(proj_seeds),
                                       A.data_ptr(), Bsum.data_ptr(), workspace.data_ptr(), nbytes, _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_debug_buckets")
    return A, Bsum


def race_attn_state_bytes(desc: RaceAttnDesc) -> int:
    return int(lib().race_attn_state_bytes(ctypes.byref(desc)))


def race_attn_state_init(desc: RaceAttnDesc, K, V, proj_seeds: Sequence[int], state=None, workspace=None, stream=None):
    """State (B, H, L, R, d+1) float32 holding the bucket statistics of the desc.N keys/values (zeros for N == 0)."""
    torch = _torch()
    shape = (desc.B, desc.H, desc.L, 1 << desc.P, desc.d + 1)
    device = K.device if K is not None else (state.device if state is not None else "cuda")
    state = torch.empty(shape, dtype=torch.float32, device=device) if state is None else state
    _check_tensor(state, desc, "state", shape, torch.float32)
    if desc.N > 0:
        _check_tensor(K, desc, "K")
        _check_tensor(V, desc, "V")
        workspace, nbytes = _workspace(desc, workspace, K.device)
        wptr = workspace.data_ptr()
    else:
        nbytes, wptr = 0, None
    st = lib().race_attn_state_init(ctypes.byref(desc), K.data_ptr() if desc.N > 0 else None,
                                    V.data_ptr() if desc.N > 0 else None, _seeds(proj_seeds), state.data_ptr(),
                                    wptr, nbytes, _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_state_init")
    return state


def race_attn_step_workspace_bytes(desc: RaceAttnDesc) -> int:
    return int(lib().race_attn_step_workspace_bytes(ctypes.byref(desc)))


def race_attn_step(desc: RaceAttnDesc, q, k, v, proj_seeds: Sequence[int], state, o=None, den=None, workspace=None,
                   stream=None):
    """One decoding step: q, k, v (B, H, d); state updated in place; returns o (B, H, d) and den (B, H).
    proj_seeds = None: the workspace (then a required argument) still holds W from an earlier step."""
    torch = _torch()
    row = (desc.B, desc.H, desc.d)
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _check_tensor(t, desc, n, row)
    _check_tensor(state, desc, "state", (desc.B, desc.H, desc.L, 1 << desc.P, desc.d + 1), torch.float32)
    o = torch.empty_like(v) if o is None else o
    den = torch.empty((desc.B, desc.H), dtype=torch.float32, device=v.device) if den is None else den
    _check_tensor(o, desc, "o", row)
    _check_tensor(den, desc, "den", (desc.B, desc.H), torch.float32)
    need = race_attn_step_workspace_bytes(desc)
    if workspace is None:
        if proj_seeds is None:
            raise ValueError("race_attn_step without seeds needs the workspace of an earlier step")
        workspace = torch.empty(need, dtype=torch.uint8, device=v.device)
    st = lib().race_attn_step(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                              _seeds(proj_seeds) if proj_seeds is not None else None,
                              state.data_ptr(), o.data_ptr(), den.data_ptr(), workspace.data_ptr(),
                              workspace.numel() * workspace.element_size(), _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_step")
    return o, den


def race_attn_calibration_copy(dst, src, stream=None) -> None:
    """Plain device copy of src into dst (equal byte sizes, a multiple of 16) by one kernel of known traffic."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src differ in size")
    st = lib().race_attn_calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_calibration_copy")


def race_attn_calibration_mfma(workgroups: int, iters: int, sink, stream=None, vector_ops: int = 0) -> int:
    """Dense bf16 MFMA loop, `vector_ops` (0, 4, 8, 16) independent vector multiplies after every matrix instruction;
    sink: float32 device tensor of workgroups * 256 elements.  Returns the flop count of the matrix instructions."""
    if sink.numel() < workgroups * 256:
        raise ValueError("sink too small")
    st = lib().race_attn_calibration_mfma(int(workgroups), int(iters), int(vector_ops), sink.data_ptr(), _stream(stream))
    if st != RACE_OK:
        raise RaceAttnError(st, "race_attn_calibration_mfma")
    return workgroups * 4 * iters * 4 * 32768


def race_attn_profile_enable(on: bool) -> None:
    lib().race_attn_profile_enable(int(bool(on)))


def race_attn_profile_read(max_entries: int = 32):
    """{kernel name: (total milliseconds, launches)} since the previous read."""
    names = (ctypes.c_char_p * max_entries)()
    ms = (ctypes.c_float * max_entries)()
    cnt = (ctypes.c_int * max_entries)()
    n = min(lib().race_attn_profile_read(max_entries, names, ms, cnt), max_entries)
    return {names[i].decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}
