"""GPU parity of the descriptor's unit-norm option (rows of Q and K divided by their Euclidean norms inside the
layer: the setting |Q_i| = |K_j| = 1 of Theorem 1's proof) against the oracle's unit_rows() in front of the layer and
unit_rows_vjp() behind its backward pass, for both kernel families, the taps and incremental decoding.

Inputs: the seeded tensors of the other parity tests with every row of Q and K stretched by its own factor, log-uniform
over [1/16, 16], so that the option has something to undo and the cotangents (which scale with 1 / |x|) span rows of
very different lengths."""
import numpy as np
import pytest
import torch

import paper_2510_04008_amd as ra
from oracle import race_oracle as ro
from paper_2510_04008_amd import synth
from paper_2510_04008_amd.synth import Workload

from parity_util import TOL, check_case, check_dbeta, desc_of, oracle_w, rel_err, run_gpu, to_f64

pytestmark = pytest.mark.gpu


def _stretched(w: Workload, seed=5):
    Q, K, V, dO = synth.make_inputs(w, "cuda")
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    for X in (Q, K):
        f = torch.exp2(torch.rand((w.B, w.H, w.N, 1), generator=gen) * 8.0 - 4.0).to("cuda")
        X.copy_((X.float() * f).to(X.dtype))
    return Q, K, V, dO


def W_(name, B, H, N, d, L, P, beta, causal, dtype, chunk=0):
    return Workload(name, B, H, N, d, L, P, beta, causal, dtype, chunk=chunk, unit_qk=True)


CASES = [
    W_("unit-generic-f32-noncausal", 1, 2, 300, 64, 4, 4, 8.0, False, "f32"),
    W_("unit-generic-f32-causal", 2, 1, 333, 64, 4, 4, 8.0, True, "f32", chunk=64),
    W_("unit-generic-bf16-odd-shape", 1, 2, 200, 96, 3, 5, 6.0, True, "bf16", chunk=64),
    W_("unit-headline-causal", 1, 2, 1000, 128, 8, 6, 8.0, True, "bf16", chunk=256),
    W_("unit-headline-noncausal", 1, 2, 777, 128, 8, 6, 8.0, False, "bf16", chunk=256),
    W_("unit-encoder-noncausal", 2, 2, 900, 64, 16, 4, 4.0, False, "bf16"),
    W_("unit-encoder-causal", 1, 2, 650, 64, 16, 4, 4.0, True, "bf16", chunk=128),
    W_("unit-padded-3x3", 1, 2, 1000, 128, 3, 3, 8.0, True, "bf16", chunk=256),
    W_("unit-padded-4x4", 1, 2, 500, 128, 4, 4, 8.0, False, "bf16"),
    W_("unit-padded-2x2", 1, 2, 700, 128, 2, 2, 8.0, True, "bf16", chunk=160),
    W_("unit-padded-6x4-d64", 1, 2, 600, 64, 6, 4, 6.0, True, "bf16", chunk=96),
    W_("unit-padded-5x5", 1, 1, 450, 128, 5, 5, 8.0, True, "bf16", chunk=128),
    W_("unit-one-tile", 1, 1, 19, 128, 8, 6, 8.0, True, "bf16"),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_forward_and_backward(w):
    check_case(w, tensors=_stretched(w))


def test_backward_on_the_forward_workspace():
    w = W_("unit-headline-saved", 1, 2, 1500, 128, 8, 6, 8.0, True, "bf16", chunk=512)
    t = _stretched(w)
    g0 = run_gpu(w, t)
    g1 = run_gpu(w, t, saved=True)
    for n in ("O", "den", "dQ", "dK", "dV"):
        assert torch.equal(g0[n], g1[n]), n


@pytest.mark.parametrize("w", [
    W_("unit-dbeta-generic", 1, 2, 200, 64, 4, 4, 2.0, True, "f32", chunk=64),
    W_("unit-dbeta-headline", 1, 2, 600, 128, 8, 6, 2.0, True, "bf16", chunk=256),
], ids=lambda w: w.name)
def test_temperature_cotangent(w):
    check_dbeta(w)


@pytest.mark.parametrize("w", [
    W_("unit-scale-generic", 1, 2, 150, 64, 4, 4, 8.0, True, "f32", chunk=64),
    W_("unit-scale-headline", 1, 2, 400, 128, 8, 6, 8.0, True, "bf16", chunk=128),
], ids=lambda w: w.name)
def test_stretching_rows_by_powers_of_four_changes_nothing_but_the_scale_of_the_cotangents(w):
    """|4^k x|^2 = 16^k |x|^2 exactly, and the reciprocal square root of a float scaled by an even power of two is
    the same mantissa: O and den come back bit-identical and dQ, dK exactly 4^-k times as large."""
    Q, K, V, dO = _stretched(w)
    g0 = run_gpu(w, (Q, K, V, dO))
    gen = torch.Generator(device="cpu")
    gen.manual_seed(11)
    kq = torch.randint(-2, 3, (w.B, w.H, w.N, 1), generator=gen).to("cuda")
    kk = torch.randint(-2, 3, (w.B, w.H, w.N, 1), generator=gen).to("cuda")
    Q2 = (Q.float() * torch.pow(4.0, kq.float())).to(Q.dtype)
    K2 = (K.float() * torch.pow(4.0, kk.float())).to(K.dtype)
    g1 = run_gpu(w, (Q2, K2, V, dO))
    assert torch.equal(g0["O"], g1["O"]) and torch.equal(g0["den"], g1["den"]) and torch.equal(g0["dV"], g1["dV"])
    assert torch.equal(g0["dQ"].float(), g1["dQ"].float() * torch.pow(4.0, kq.float()))
    assert torch.equal(g0["dK"].float(), g1["dK"].float() * torch.pow(4.0, kk.float()))


@pytest.mark.parametrize("w", [
    W_("unit-tangent-generic", 1, 1, 120, 64, 4, 4, 8.0, True, "f32", chunk=64),
    W_("unit-tangent-headline", 1, 2, 300, 128, 8, 6, 8.0, True, "bf16", chunk=128),
], ids=lambda w: w.name)
def test_cotangents_have_no_component_along_the_row(w):
    """O does not depend on a row's length, so dQ_i . Q_i = dK_j . K_j = 0; what the device leaves is the rounding
    of its stored cotangent (2^-9 per element in bf16, 2^-24 in fp32), not a systematic radial part."""
    g = run_gpu(w, _stretched(w))
    ulp = 2.0 ** -8 if w.dtype == "bf16" else 2.0 ** -20
    for X, dX in ((g["Q"], g["dQ"]), (g["K"], g["dK"])):
        X, dX = to_f64(X), to_f64(dX)
        radial = np.abs((X * dX).sum(axis=-1))
        bound = ulp * np.sqrt((X * X).sum(axis=-1)) * np.sqrt((dX * dX).sum(axis=-1)) + 1e-30
        assert (radial <= bound).all(), float((radial / bound).max())


def test_zero_rows_stay_zero_and_everything_stays_finite():
    w = W_("unit-zero-rows", 1, 2, 200, 128, 8, 6, 8.0, True, "bf16", chunk=64)
    Q, K, V, dO = _stretched(w)
    Q[:, :, 7] = 0
    K[:, :, 50] = 0
    K[:, :, 199] = 0
    g = run_gpu(w, (Q, K, V, dO))
    W = oracle_w(w, g["seeds"])
    O, den = ro.forward(ro.unit_rows(to_f64(Q)), ro.unit_rows(to_f64(K)), to_f64(V), list(W), w.sharpening, w.L, w.P, True)
    assert rel_err(g["O"], O) < TOL["bf16"] and rel_err(g["den"], den) < TOL["bf16"]
    for n in ("dQ", "dK", "dV"):
        assert torch.isfinite(g[n].float()).all(), n


@pytest.mark.parametrize("w", [
    W_("unit-taps-generic", 1, 2, 90, 64, 4, 4, 8.0, False, "f32"),
    W_("unit-taps-headline", 1, 2, 130, 128, 8, 6, 8.0, False, "bf16"),
    W_("unit-taps-padded", 1, 2, 70, 128, 3, 3, 8.0, False, "bf16"),
], ids=lambda w: w.name)
def test_taps(w):
    Q, K, V, _ = _stretched(w)
    seeds = synth.projection_seeds(w)
    W = oracle_w(w, seeds)
    d = desc_of(w)
    codes, phi = ra.race_attn_debug_hash(d, K, seeds, want_phi=True)
    A, Bsum = ra.race_attn_debug_buckets(d, K, V, seeds)
    torch.cuda.synchronize()
    Kh, Vh = ro.unit_rows(to_f64(K)), to_f64(V)
    tol = TOL[w.dtype]
    for b in range(w.B):
        for h in range(w.H):
            ref = ro.soft_hash(Kh[b, h], W[h], w.sharpening, w.L, w.P)
            assert np.abs(to_f64(phi[b, h]).reshape(ref.shape) - ref).max() < tol
            z = ro.project(Kh[b, h], W[h], w.L, w.P)
            clear = np.abs(z).min(axis=2) > 2.0 ** -16 * np.linalg.norm(W[h], axis=1).max()
            got = codes[b, h].cpu().numpy().astype(np.int64)
            assert np.array_equal(got[clear], ro.hard_codes(Kh[b, h], W[h], w.L, w.P)[clear])
            rA, rB = ro.bucket_statistics(Kh[b, h], Vh[b, h], W[h], w.sharpening, w.L, w.P)
            assert rel_err(A[b, h], rA.reshape(to_f64(A[b, h]).shape)) < tol
            assert rel_err(Bsum[b, h], rB) < tol


@pytest.mark.parametrize("w", [
    W_("unit-decode-generic", 2, 1, 40, 64, 4, 4, 8.0, True, "f32"),
    W_("unit-decode-headline", 1, 2, 300, 128, 8, 6, 8.0, True, "bf16", chunk=128),
], ids=lambda w: w.name)
def test_decoding_steps(w):
    Q, K, V, _ = _stretched(w)
    seeds = synth.projection_seeds(w)
    W = oracle_w(w, seeds)
    n0 = w.N - 12                                                     # prefill, then token by token
    dpre = ra.make_desc(w.B, w.H, n0, w.d, w.L, w.P, w.sharpening, True, desc_of(w).dtype, w.chunk, unit_qk=True)
    state = ra.race_attn_state_init(dpre, K[:, :, :n0].contiguous(), V[:, :, :n0].contiguous(), seeds)
    outs, dens = [], []
    for t in range(n0, w.N):
        o, dn = ra.race_attn_step(dpre, Q[:, :, t].contiguous(), K[:, :, t].contiguous(), V[:, :, t].contiguous(), seeds, state)
        outs.append(o.clone()); dens.append(dn.clone())
    torch.cuda.synchronize()
    O, den = ro.forward(ro.unit_rows(to_f64(Q)), ro.unit_rows(to_f64(K)), to_f64(V), list(W), w.sharpening, w.L, w.P, True)
    assert rel_err(torch.stack(outs, dim=2), O[:, :, n0:]) < TOL[w.dtype]
    assert rel_err(torch.stack(dens, dim=2), den[:, :, n0:]) < TOL[w.dtype]


def test_hard_hash_ignores_the_option():
    """sign(W x / |x|) = sign(W x): with the hard hash the option changes nothing."""
    base = Workload("unit-hard", 1, 2, 500, 128, 8, 6, float("inf"), True, "bf16", chunk=128)
    Q, K, V, _ = _stretched(base)
    seeds = synth.projection_seeds(base)
    O0, den0 = ra.race_attn_fwd(desc_of(base), Q, K, V, seeds)
    unit = Workload("unit-hard", 1, 2, 500, 128, 8, 6, float("inf"), True, "bf16", chunk=128, unit_qk=True)
    O1, den1 = ra.race_attn_fwd(desc_of(unit), Q, K, V, seeds)
    torch.cuda.synchronize()
    assert torch.equal(O0, O1) and torch.equal(den0, den1)
