"""GPU parity of the hard-hash layer (Section 3.3's h(x) = sign(W x); temperature = +infinity at the C ABI)
against the oracle's counter form, for both kernel families, the taps and incremental decoding.

The bucket of a token is decided by the signs of its projections.  The device accumulates the dot products in
fp32 in an order of its own, so a projection inside the rounding band of the dot product could land on the other
side; such rows are replaced (by a row of the same head that is clear of every hyperplane) before either side
sees the inputs, and both sides then take the same decisions.
"""
import numpy as np
import pytest
import torch

import paper_2510_04008_amd as ra
from oracle import race_oracle as ro
from paper_2510_04008_amd import synth
from paper_2510_04008_amd.synth import Workload

from parity_util import TOL, desc_of, oracle_w, rel_err, to_f64

pytestmark = pytest.mark.gpu
INF = float("inf")


def _clear_of_hyperplanes(X, W, L, P):
    """X (B, H, N, d) device tensor, W (H, L*P, d): rows whose projection on any hyperplane lies within
    2^-16 |x| |w| of zero are overwritten with the first row of the same (batch, head) that is clear."""
    Xh = to_f64(X)
    replaced = 0
    for b in range(Xh.shape[0]):
        for h in range(Xh.shape[1]):
            z = Xh[b, h] @ W[h].T
            tau = 2.0 ** -16 * np.linalg.norm(Xh[b, h], axis=1)[:, None] * np.linalg.norm(W[h], axis=1)[None, :]
            bad = (np.abs(z) <= tau).any(axis=1)
            good = int(np.flatnonzero(~bad)[0])
            idx = torch.from_numpy(np.flatnonzero(bad)).to(X.device)
            if bad.any():
                X[b, h, idx] = X[b, h, good].clone()
            replaced += int(bad.sum())
    return replaced


def _check_counts(den, ref, L):
    """Den is a number of collisions divided by L: the count comes back exactly, the quotient to fp32 rounding."""
    got = to_f64(den)
    assert np.array_equal(np.rint(got * L), np.rint(ref * L))
    assert np.all(np.abs(got - ref) <= 2.0 ** -22 * ref)


def _inputs(w):
    Q, K, V, dO = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    W = oracle_w(w, seeds)
    n = _clear_of_hyperplanes(Q, W, w.L, w.P) + _clear_of_hyperplanes(K, W, w.L, w.P)
    return Q, K, V, seeds, W, n


CASES = [
    Workload("hard-headline-causal", 1, 2, 1000, 128, 8, 6, INF, True, "bf16", normalize_qk=True, chunk=256),
    Workload("hard-headline-noncausal", 1, 2, 1000, 128, 8, 6, INF, False, "bf16", normalize_qk=True, chunk=256),
    Workload("hard-headline-raw", 2, 2, 777, 128, 8, 6, INF, True, "bf16", chunk=256),
    Workload("hard-few-keys", 1, 2, 5, 128, 8, 6, INF, False, "bf16"),            # empty buckets: den = 0, O = 0
    Workload("hard-encoder", 2, 2, 900, 64, 16, 4, INF, False, "bf16"),
    Workload("hard-padded-3x3", 1, 2, 1000, 128, 3, 3, INF, True, "bf16", normalize_qk=True, chunk=256),
    # the paper's grid shapes (padded execution on the small compiled shapes)
    Workload("hard-counters-4x4", 1, 2, 1500, 128, 4, 4, INF, True, "bf16", normalize_qk=True, chunk=512),
    Workload("hard-counters-4x4-noncausal", 2, 2, 777, 128, 4, 4, INF, False, "bf16", chunk=256),
    Workload("hard-counters-2x2", 1, 3, 1000, 128, 2, 2, INF, True, "bf16", chunk=128),
    Workload("hard-counters-d64", 1, 2, 900, 64, 4, 4, INF, True, "bf16", normalize_qk=True, chunk=160),
    Workload("hard-counters-one-token", 1, 1, 1, 128, 4, 4, INF, True, "bf16"),
    Workload("hard-generic-f32", 1, 1, 300, 64, 4, 4, INF, True, "f32", chunk=64),
    Workload("hard-generic-f32-noncausal", 1, 2, 200, 64, 4, 4, INF, False, "f32"),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_forward_equals_the_counter_form(w):
    Q, K, V, seeds, W, replaced = _inputs(w)
    O, den = ra.race_attn_fwd(desc_of(w), Q, K, V, seeds)
    torch.cuda.synchronize()
    Qh, Kh, Vh = to_f64(Q), to_f64(K), to_f64(V)
    rO, rden = np.empty_like(Qh), np.empty(Qh.shape[:3])
    for b in range(w.B):
        for h in range(w.H):
            rO[b, h], rden[b, h] = ro.forward_hard(Qh[b, h], Kh[b, h], Vh[b, h], W[h], w.L, w.P, w.causal)
    _check_counts(den, rden, w.L)
    e = rel_err(O, rO)
    print("%s: family=%d rows replaced %d, empty queries %d, O=%.2e" %
          (w.name, ra.race_attn_kernel_family(desc_of(w)), replaced, int((rden == 0).sum()), e), flush=True)
    assert e < TOL[w.dtype]
    assert (to_f64(O)[rden == 0] == 0).all()
    if w.name == "hard-few-keys":
        assert (rden == 0).any()


def test_taps_count_keys_and_mark_one_corner():
    w = Workload("hard-taps", 1, 2, 1500, 128, 8, 6, INF, True, "bf16", normalize_qk=True, chunk=512)
    Q, K, V, seeds, W, _ = _inputs(w)
    d = desc_of(w)
    A, Bsum = ra.race_attn_debug_buckets(d, K, V, seeds)
    codes, phi = ra.race_attn_debug_hash(d, K, seeds, want_phi=True)
    torch.cuda.synchronize()
    Kh, Vh = to_f64(K), to_f64(V)
    for h in range(w.H):
        ck = ro.hard_codes(Kh[0, h], W[h], w.L, w.P)
        assert np.array_equal(codes[0, h].cpu().numpy().astype(np.int64), ck)
        onehot = np.zeros((w.N, w.L, 1 << w.P))
        np.put_along_axis(onehot, ck[:, :, None], 1.0, axis=2)
        assert np.array_equal(phi[0, h].cpu().numpy().reshape(onehot.shape), onehot)
        counts = onehot.sum(axis=0)
        assert np.array_equal(to_f64(A[0, h]), counts)                 # the mass of a bucket is its number of keys
        sums = np.einsum("nlr,nc->lrc", onehot, Vh[0, h])
        assert rel_err(Bsum[0, h], sums) < 1e-5                        # fp32 sums of bf16 values


@pytest.mark.parametrize("w", [
    Workload("hard-decode-mfma", 1, 2, 40, 128, 8, 6, INF, True, "bf16", normalize_qk=True),
    Workload("hard-decode-generic", 2, 1, 30, 64, 4, 4, INF, True, "f32"),
], ids=lambda w: w.name)
def test_decoding_steps(w):
    Q, K, V, seeds, W, _ = _inputs(w)
    d = desc_of(w)
    n0 = w.N // 2                                                     # prefill, then token by token
    dpre = ra.make_desc(w.B, w.H, n0, w.d, w.L, w.P, INF, True, d.dtype, 0)
    state = ra.race_attn_state_init(dpre, K[:, :, :n0].contiguous(), V[:, :, :n0].contiguous(), seeds)
    outs, dens = [], []
    for t in range(n0, w.N):
        o, dn = ra.race_attn_step(d, Q[:, :, t].contiguous(), K[:, :, t].contiguous(), V[:, :, t].contiguous(), seeds, state)
        outs.append(o.clone()); dens.append(dn.clone())
    torch.cuda.synchronize()
    got_O = torch.stack(outs, dim=2)
    got_den = torch.stack(dens, dim=2)
    Qh, Kh, Vh = to_f64(Q), to_f64(K), to_f64(V)
    for b in range(w.B):
        for h in range(w.H):
            rO, rden = ro.forward_hard(Qh[b, h], Kh[b, h], Vh[b, h], W[h], w.L, w.P, True)
            _check_counts(got_den[b, h], rden[n0:], w.L)
            assert rel_err(got_O[b, h], rO[n0:]) < TOL[w.dtype]
