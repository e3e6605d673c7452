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
