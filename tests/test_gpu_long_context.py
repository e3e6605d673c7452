"""The long-context configurations at full size, in the launch configuration the benchmark times (forward, then the
backward pass on the forward's workspace), against the fp64 oracle.

The oracle walks the sequence slice by slice with carried bucket statistics (oracle/stream.py: equal to a whole run
bit for bit, pinned on the CPU), reading the same device buffers the kernels read, so host memory stays bounded:
  * a PREFIX reaching past the third scan-segment boundary: O, Den and dQ of a causal layer depend on no later token;
  * a TAIL window across the last segment boundaries: dK and dV depend on the tokens behind them only once O and Den
    are given (the suffix statistics of the read-out cotangents); this is also the check of row addressing beyond
    2^31 elements, which constant-value invariants cannot see;
  * where the oracle's speed allows, every token: O and Den over all of configuration 4, all five tensors at 2^20
    tokens of the headline shape with the default plan of 128 segments per head;
  * properties that hold at any size (V = 1 gives O = 1; sum of dV = sum of dO).
Each comparison reports, and asserts, the tensor-wide max-ratio of the tolerance statement, the relative l2 error and
the max-ratio per block of 1024 tokens.
"""
import os

import numpy as np
import pytest
import torch

import paper_2510_04008_amd as ra
from oracle import stream as oracle_stream
from paper_2510_04008_amd import synth

from parity_util import BLOCK_FACTOR, TOL, ErrAcc, desc_of, oracle_w, to_f64

BLK_TOL = {n: BLOCK_FACTOR * TOL["bf16"] for n in ("dQ", "dK", "dV")}

pytestmark = pytest.mark.gpu

SLICE = 65536


def _pull(t, a, b):
    return to_f64(t[:, :, a:b])


def _report(name, what, accs):
    print("%s %s: " % (name, what) + "  ".join("%s[%s]" % kv for kv in accs.items()), flush=True)


def _assert(accs, tol, blk_tol, what):
    for n, e in accs.items():
        assert e.linf < tol, (what, n, "linf", e.linf)
        assert e.l2 < tol, (what, n, "l2", e.l2)
        assert e.blk < blk_tol.get(n, tol), (what, n, "blk", e.blk, e.worst_block)


def forward_sweep(w, t, fwd, W, n_tokens, keep_windows=()):
    """Oracle forward over tokens [0, n_tokens) in slices; compares the kernels' O and Den on the fly.  keep_windows:
    token ranges (a, b) whose oracle O and Den are returned, rounded to the layer's storage types (what a caller of the
    backward pass holds after an exact forward pass), as {(a, b): (O bf16 tensor, den fp32 tensor)}."""
    st = oracle_stream.new_state(w.B, w.H, w.L, w.P, w.d)
    accs = {n: ErrAcc() for n in ("O", "den")}
    kept = {win: ([], []) for win in keep_windows}
    min_den = np.inf
    cuts = sorted(set([0, n_tokens] + list(range(0, n_tokens, SLICE)) + [x for win in keep_windows for x in win if x <= n_tokens]))
    for a, b in zip(cuts[:-1], cuts[1:]):
        O, den = oracle_stream.forward_slice(_pull(t["Q"], a, b), _pull(t["K"], a, b), _pull(t["V"], a, b), W,
                                             w.sharpening, w.L, w.P, st)
        min_den = min(min_den, float(den.min()))
        accs["O"].update(fwd["O"][:, :, a:b], O, a)
        accs["den"].update(fwd["den"][:, :, a:b].unsqueeze(-1), den[..., None], a)
        for (wa, wb), (lo, ld) in kept.items():
            if wa <= a and b <= wb:
                lo.append(torch.from_numpy(O).to(torch.float32).to(torch.bfloat16))
                ld.append(torch.from_numpy(den).to(torch.float32))
    assert min_den > 1e-30
    return accs, {win: (torch.cat(lo, dim=2), torch.cat(ld, dim=2)) for win, (lo, ld) in kept.items()}


def query_sweep(w, t, O_in, den_in, dQ, W, n_tokens):
    """Oracle query pass of the backward pass over tokens [0, n_tokens), given O_in, den_in (device tensors, the same
    the kernels were given); compares dQ."""
    st = oracle_stream.new_state(w.B, w.H, w.L, w.P, w.d)
    acc = ErrAcc()
    for a in range(0, n_tokens, SLICE):
        b = min(n_tokens, a + SLICE)
        ref = oracle_stream.backward_slice(_pull(t["Q"], a, b), _pull(t["K"], a, b), _pull(t["V"], a, b), W, w.sharpening,
                                           w.L, w.P, _pull(O_in, a, b), to_f64(den_in[:, :, a:b]), _pull(t["dO"], a, b),
                                           prefix_state=st)[0]
        acc.update(dQ[:, :, a:b], ref, a)
    return {"dQ": acc}


def keyvalue_sweep(w, t, O_in, den_in, dK, dV, W, start):
    """Oracle key/value pass over tokens [start, N) in slices from the far end, given O_in, den_in; compares dK, dV."""
    st = oracle_stream.new_state(w.B, w.H, w.L, w.P, w.d)
    accs = {n: ErrAcc() for n in ("dK", "dV")}
    edges = list(range(start, w.N, SLICE)) + [w.N]
    for a, b in reversed(list(zip(edges[:-1], edges[1:]))):
        _, rK, rV = oracle_stream.backward_slice(_pull(t["Q"], a, b), _pull(t["K"], a, b), _pull(t["V"], a, b), W,
                                                 w.sharpening, w.L, w.P, _pull(O_in, a, b), to_f64(den_in[:, :, a:b]),
                                                 _pull(t["dO"], a, b), suffix_state=st)
        accs["dK"].update(dK[:, :, a:b], rK, a)
        accs["dV"].update(dV[:, :, a:b], rV, a)
    return accs


def size_free_properties(w, g, Q, K, V, dO):
    for n in ("O", "den", "dQ", "dK", "dV"):
        assert torch.isfinite(g[n][:, :, ::4097].float()).all(), n
    assert (g["den"][:, :, ::1000] > 0).all()
    # rows of the attention matrix sum to one: total value gradient equals total upstream gradient
    tot = torch.zeros((w.B, w.H, w.d), dtype=torch.float64, device="cuda")
    ref = torch.zeros_like(tot)
    step = 1 << 20
    for s in range(0, w.N, step):
        tot += g["dV"][:, :, s:s + step].double().sum(dim=2)
        ref += dO[:, :, s:s + step].double().sum(dim=2)
    scale = dO.float().abs().max().item() * (w.N ** 0.5)
    assert (tot - ref).abs().max().item() < 2e-2 * scale
    # constant values come back as that constant at every position
    V.fill_(1.0)
    O1, _ = ra.race_attn_fwd(desc_of(w), Q, K, V, synth.projection_seeds(w))
    torch.cuda.synchronize()
    for s in range(0, w.N, step):
        assert (O1[:, :, s:s + step].float() - 1.0).abs().max().item() < 1e-2


def _long_context(w, forward="prefix", backward="windows"):
    """forward: "prefix" (O, Den up to past the third segment boundary) or "all" (every token);
    backward: "windows" (dQ on that prefix; dK, dV on a tail window) or "all" (every token).
    The backward pass is a function of (Q, K, V, O, Den, dO).  Wherever the oracle's forward sweep reaches, the kernels'
    backward pass and the oracle's are both given the ORACLE's O and Den rounded to bf16 / fp32 (the kernels' own O and
    Den are checked against the oracle's separately); where it does not reach (the tail of the 12 M-token run, whose
    forward results depend on every earlier token), both are given the kernels' O and Den of those rows."""
    assert ra.race_attn_kernel_family(desc_of(w)) == 2
    d = desc_of(w)
    seg = ra.race_attn_segment_tokens(d)
    nseg = (w.N + seg - 1) // seg
    seeds = synth.projection_seeds(w)
    Q, K, V, dO = synth.make_inputs(w, "cuda", on_device_rng=True)
    t = dict(Q=Q, K=K, V=V, dO=dO)
    W = oracle_w(w, seeds)
    tol = TOL["bf16"]
    print("%s: N=%d, %d segments of %d tokens per head" % (w.name, w.N, nseg, seg), flush=True)
    ws = torch.empty(ra.race_attn_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    O, den = ra.race_attn_fwd(d, Q, K, V, seeds, workspace=ws)
    torch.cuda.synchronize()

    n_pre = min(w.N, 3 * seg + 1024)                          # past the third segment boundary
    n_tail = w.N if backward == "all" else min(w.N, max(131072, seg + 32768))   # across the last boundary (four of them at 4 M)
    n_fwd = w.N if (forward == "all" or backward == "all") else n_pre
    pre_win = (0, w.N) if backward == "all" else (0, n_pre)
    tail_win = (w.N - n_tail, w.N)
    wins = [pre_win] + ([tail_win] if n_fwd == w.N and tail_win != pre_win else [])
    accs, kept = forward_sweep(w, t, dict(O=O, den=den), W, n_fwd, wins)
    _report(w.name, "tokens [0, %d)" % n_fwd, accs)
    _assert(accs, tol, {}, "forward")

    # forward results handed to the backward pass: the oracle's (rounded) on the windows it reached
    O_in, den_in = O.clone(), den.clone()
    for (a, b), (Ow, dw) in kept.items():
        O_in[:, :, a:b] = Ow.cuda()
        den_in[:, :, a:b] = dw.cuda()
    fed_tail = "the oracle's" if tail_win in kept or pre_win == (0, w.N) else "the kernels'"
    del kept
    dQ, dK, dV = ra.race_attn_bwd_saved(d, Q, K, V, O_in, den_in, dO, seeds, ws)
    torch.cuda.synchronize()
    accs = query_sweep(w, t, O_in, den_in, dQ, W, pre_win[1])
    _report(w.name, "tokens [0, %d), given the oracle's O and Den" % pre_win[1], accs)
    _assert(accs, tol, BLK_TOL, "query pass")
    accs = keyvalue_sweep(w, t, O_in, den_in, dK, dV, W, tail_win[0])
    _report(w.name, "tokens [%d, %d), given %s O and Den" % (tail_win[0], w.N, fed_tail), accs)
    _assert(accs, tol, BLK_TOL, "key/value pass")

    size_free_properties(w, dict(O=O, den=den, dQ=dQ, dK=dK, dV=dV), Q, K, V, dO)


def test_config4_causal_4m_tokens():
    # O and Den against the oracle at every one of the 4 194 304 tokens; dQ across the first three segment boundaries;
    # dK, dV across the last four, from the oracle's own O and Den
    _long_context(synth.C4, forward="all")


def test_config5_causal_12m_tokens():
    # O, Den, dQ across the first three segment boundaries (295 936 tokens); dK, dV on the last 131 072 tokens (element
    # offsets up to 6.4e9), from the kernels' O and Den of those rows
    _long_context(synth.C5)


def test_headline_shape_1m_tokens_every_token_all_five_tensors():
    w = synth.C5.scaled(1 << 20, "C5-shape-1M")
    assert (w.N + ra.race_attn_segment_tokens(desc_of(w)) - 1) // ra.race_attn_segment_tokens(desc_of(w)) == 128
    _long_context(w, forward="all", backward="all")


@pytest.mark.parametrize("w", [synth.G22, synth.G44], ids=lambda w: w.name)
def test_paper_grid_1m_tokens(w):
    # the paper's own scaling grid at N = 2^20, on the padded 64-row shape, in the benchmark's launch configuration
    _long_context(w)


def test_paper_grid_16m_tokens():
    # (P, L) = (4, 4) at 2^24 tokens, beyond the 12 M the paper reports for its own runs: 17 GB per tensor, element offsets
    # up to 8.6e9; O, Den, dQ across the first three segment boundaries, dK, dV across the last
    _long_context(synth.G44.scaled(1 << 24, "G44-causal-bf16-16M"))
