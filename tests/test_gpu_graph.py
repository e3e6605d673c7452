"""The forward and backward passes are plain stream work (kernels and one pinned host-to-device copy): they can be
captured into a HIP graph and replayed.  Every replay is compared with the eager result, with eager work and
synchronisations between the replays."""
import pytest
import torch

import paper_2510_04008_amd as ra
from paper_2510_04008_amd import synth
from paper_2510_04008_amd.synth import Workload

from parity_util import desc_of

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("w", [
    Workload("graph-bf16", 1, 2, 1500, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True, chunk=256),
    Workload("graph-f32", 1, 2, 300, 64, 4, 4, 8.0, True, "f32", chunk=64),
], ids=lambda w: w.name)
def test_forward_backward_replay_from_a_graph(w):
    Q, K, V, dO = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    d = desc_of(w)
    ws = torch.empty(ra.race_attn_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    O, den = torch.empty_like(V), torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dbeta = torch.empty((w.B, w.H), dtype=torch.float32, device="cuda")

    def step():
        ra.race_attn_fwd(d, Q, K, V, seeds, O=O, den=den, workspace=ws)
        ra.race_attn_bwd_beta(d, Q, K, V, O, den, dO, seeds, dQ=dQ, dK=dK, dV=dV, dbeta=dbeta, workspace=ws)

    step()                                   # eager: also creates the cached projection image before capture
    torch.cuda.synchronize()
    want = [t.clone() for t in (O, den, dQ, dK, dV, dbeta)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    for rep in range(3):
        for t in (O, den, dQ, dK, dV, dbeta):
            t.fill_(float("nan")) if t.dtype == torch.float32 else t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((O, den, dQ, dK, dV, dbeta), want):
            assert torch.equal(got, ref), "replay %d differs from the eager result" % rep
        # eager work between the replays
        step()
        torch.cuda.synchronize()
        for got, ref in zip((O, den, dQ, dK, dV, dbeta), want):
            assert torch.equal(got, ref)


@pytest.mark.parametrize("w", [
    Workload("graph-decode-bf16", 2, 2, 12, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True),
    Workload("graph-decode-f32", 1, 2, 12, 64, 4, 4, 8.0, True, "f32"),
], ids=lambda w: w.name)
def test_decoding_steps_replay_from_a_graph(w):
    """A serving loop without host work per token: a run of race_attn_step calls (the state carried in place) is
    captured once and replayed; every replay reproduces the eager run from the same starting state bit for bit."""
    Q, K, V, _ = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    d = desc_of(w)
    q, k, v = (t.transpose(1, 2).transpose(0, 1).contiguous() for t in (Q, K, V))     # (N, B, H, d): one row set per step
    d0 = ra.make_desc(w.B, w.H, 0, w.d, w.L, w.P, w.sharpening, True, d.dtype, 0)
    start = ra.race_attn_state_init(d0, None, None, seeds)
    state = start.clone()
    ws = torch.empty(max(ra.race_attn_step_workspace_bytes(d), 256), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(q)
    den = torch.empty((w.N, w.B, w.H), dtype=torch.float32, device="cuda")

    def run():
        for t in range(w.N):
            ra.race_attn_step(d, q[t], k[t], v[t], seeds, state, o=out[t], den=den[t], workspace=ws)

    run()
    torch.cuda.synchronize()
    want = [out.clone(), den.clone(), state.clone()]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    state.copy_(start)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()
    for rep in range(3):
        state.copy_(start)
        out.zero_(); den.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((out, den, state), want):
            assert torch.equal(got, ref), "replay %d differs from the eager run" % rep
        state.copy_(start)
        run()                                 # eager work between the replays
        torch.cuda.synchronize()
        for got, ref in zip((out, den, state), want):
            assert torch.equal(got, ref)
    # per-step time of a replay (no host work between the steps)
    state.copy_(start)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); graph.replay(); e1.record()
    torch.cuda.synchronize()
    print("%s: %.1f us per decoding step from the graph" % (w.name, e0.elapsed_time(e1) * 1e3 / w.N), flush=True)
