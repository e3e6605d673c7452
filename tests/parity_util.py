"""Shared helpers of the GPU parity tests: run the HIP path through the C-ABI binding, run the oracle on
the same (rounded) inputs, and compare with the error measure of the build's tolerance statement."""
from __future__ import annotations

import numpy as np
import torch

import paper_2510_04008_amd as ra
from oracle import race_oracle as ro
from oracle import stream as oracle_stream
from paper_2510_04008_amd import synth

# max |gpu - oracle| / max |oracle| per output tensor
TOL = {"f32": 1e-4, "bf16": 2e-2}


def desc_of(w: synth.Workload):
    return ra.make_desc(w.B, w.H, w.N, w.d, w.L, w.P, w.sharpening, w.causal,
                        ra.RACE_F32 if w.dtype == "f32" else ra.RACE_BF16, w.chunk, w.unit_qk)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def oracle_w(w: synth.Workload, seeds):
    return np.stack([ro.expand_projection(s, w.L, w.P, w.d, round_bf16=(w.dtype == "bf16")) for s in seeds])


def rel_err(gpu: torch.Tensor, ref: np.ndarray, floor: float = 0.0) -> float:
    """floor: lower bound of the scale, for tensors that are zero in exact arithmetic."""
    g = to_f64(gpu)
    assert np.isfinite(g).all(), "non-finite values in GPU result"
    scale = max(np.abs(ref).max(), floor)
    return float(np.abs(g - ref).max() / (scale if scale > 0 else 1.0))


def run_gpu(w: synth.Workload, tensors=None, seeds=None, saved=False):
    """One forward and one backward pass through the C ABI.  saved: the backward pass reads the workspace the
    forward pass left behind (race_attn_bwd_saved), the pair of calls the benchmark times."""
    Q, K, V, dO = tensors if tensors is not None else synth.make_inputs(w, "cuda")
    seeds = seeds if seeds is not None else synth.projection_seeds(w)
    d = desc_of(w)
    if saved:
        ws = torch.empty(ra.race_attn_workspace_bytes(d), dtype=torch.uint8, device="cuda")
        O, den = ra.race_attn_fwd(d, Q, K, V, seeds, workspace=ws)
        dQ, dK, dV = ra.race_attn_bwd_saved(d, Q, K, V, O, den, dO, seeds, ws)
    else:
        O, den = ra.race_attn_fwd(d, Q, K, V, seeds)
        dQ, dK, dV = ra.race_attn_bwd(d, Q, K, V, O, den, dO, seeds)
    torch.cuda.synchronize()
    return dict(Q=Q, K=K, V=V, dO=dO, O=O, den=den, dQ=dQ, dK=dK, dV=dV, seeds=seeds)


def run_oracle(w: synth.Workload, g):
    W = oracle_w(w, g["seeds"])
    Q, K, V, dO = (to_f64(g[n]) for n in ("Q", "K", "V", "dO"))
    # the unit-norm option is the map x -> x / |x| in front of the layer and its chain rule behind the backward pass
    Qu, Ku = (ro.unit_rows(Q), ro.unit_rows(K)) if w.unit_qk else (Q, K)
    O, den = oracle_stream.forward(Qu, Ku, V, W, w.sharpening, w.L, w.P, w.causal)
    # the backward pass is a function of (Q, K, V, O, den, dO); feed it the oracle's own O and den
    dQ, dK, dV = oracle_stream.backward(Qu, Ku, V, W, w.sharpening, w.L, w.P, w.causal, O, den, dO)
    if w.unit_qk:
        dQ, dK = ro.unit_rows_vjp(Q, dQ), ro.unit_rows_vjp(K, dK)
    return dict(O=O, den=den, dQ=dQ, dK=dK, dV=dV)


def check_case(w: synth.Workload, tensors=None, tol=None, verbose=True, floors=None):
    tol = tol or TOL[w.dtype]
    floors = floors or {}
    g = run_gpu(w, tensors)
    r = run_oracle(w, g)
    errs = {n: rel_err(g[n], r[n], floors.get(n, 0.0)) for n in ("O", "den", "dQ", "dK", "dV")}
    if verbose:
        print("%s: family=%d " % (w.name, ra.race_attn_kernel_family(desc_of(w))) +
              " ".join("%s=%.2e" % kv for kv in errs.items()), flush=True)
    assert r["den"].min() > 1e-30
    for n, e in errs.items():
        assert e < tol, "%s: %s rel err %.3e >= %.1e" % (w.name, n, e, tol)
    return g, r, errs


def check_dbeta(w: synth.Workload, tol=None, verbose=True, scale="max"):
    """Cotangent of the temperature per (batch, head) from race_attn_bwd_beta against the oracle; also checks
    that asking for it leaves dQ, dK, dV bit-identical.  scale "max": the error measure of the tensors,
    max |gpu - oracle| / max |oracle|, for inputs whose terms do not cancel much.  scale "l1": relative to
    the sum of the absolute values of the terms (per batch and head), for inputs where tens of thousands of
    terms of both signs cancel to a small sum and every term carries the path's rounding."""
    tol = tol or TOL[w.dtype]
    g = run_gpu(w)
    d = desc_of(w)
    dQ, dK, dV, dbeta = ra.race_attn_bwd_beta(d, g["Q"], g["K"], g["V"], g["O"], g["den"], g["dO"], g["seeds"])
    torch.cuda.synchronize()
    for a, b in ((dQ, g["dQ"]), (dK, g["dK"]), (dV, g["dV"])):
        assert torch.equal(a, b)
    W = oracle_w(w, g["seeds"])
    Q, K, V, dO = (to_f64(g[n]) for n in ("Q", "K", "V", "dO"))
    if w.unit_qk:
        Q, K = ro.unit_rows(Q), ro.unit_rows(K)
    O, den = oracle_stream.forward(Q, K, V, W, w.sharpening, w.L, w.P, w.causal)
    *_, ref = oracle_stream.backward(Q, K, V, W, w.sharpening, w.L, w.P, w.causal, O, den, dO, with_beta=True)
    got = to_f64(dbeta)
    assert np.isfinite(got).all()
    if scale == "l1":
        l1 = np.array([[ro.beta_cotangent_l1(Q[b, h], K[b, h], V[b, h], W[h], w.sharpening, w.L, w.P, w.causal, dO[b, h])
                        for h in range(w.H)] for b in range(w.B)])
        assert (l1 >= np.abs(ref) * (1 - 1e-9)).all()
        err = float((np.abs(got - ref) / l1).max())
        note = "relative to the terms' l1 norm %.3e (|dbeta| %.3e)" % (l1.max(), np.abs(ref).max())
    else:
        err = float(np.abs(got - ref).max() / np.abs(ref).max())
        note = "relative to max |dbeta| %.3e" % np.abs(ref).max()
    if verbose:
        print("%s: dbeta err %.2e %s" % (w.name, err, note), flush=True)
    assert err < tol, "%s: dbeta err %.3e >= %.1e (%s)" % (w.name, err, tol, note)
    return dbeta, ref
