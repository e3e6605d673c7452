"""GPU parity of incremental decoding (the loop body of Algorithm 2 with the bucket statistics as the carried
state) against the fp64 oracle, through the C ABI: from an empty state, and after a prefill by either kernel family."""
import numpy as np
import pytest
import torch

import paper_2510_04008_amd as ra
from oracle import race_oracle as ro
from paper_2510_04008_amd import synth
from paper_2510_04008_amd.synth import Workload

from parity_util import TOL, desc_of, oracle_w, to_f64

pytestmark = pytest.mark.gpu


def _decode_against_oracle(w: Workload, n_prefill: int, n_steps: int):
    """Prefill the first n_prefill tokens with race_attn_state_init, then feed the next n_steps tokens one by one."""
    total = Workload(w.name, w.B, w.H, n_prefill + n_steps, w.d, w.L, w.P, w.sharpening, True, w.dtype,
                     normalize_qk=w.normalize_qk, chunk=w.chunk)
    Q, K, V, _ = synth.make_inputs(total, "cuda")
    seeds = synth.projection_seeds(total)
    W = oracle_w(total, seeds)
    pre = Workload(w.name, w.B, w.H, n_prefill, w.d, w.L, w.P, w.sharpening, True, w.dtype, chunk=w.chunk)
    dp = desc_of(pre)
    state = ra.race_attn_state_init(dp, K[:, :, :n_prefill].contiguous() if n_prefill else None,
                                    V[:, :, :n_prefill].contiguous() if n_prefill else None, seeds)
    assert state.numel() * 4 == ra.race_attn_state_bytes(dp)
    # oracle: the causal forward over the whole sequence gives every step's expected output
    Qd, Kd, Vd = to_f64(Q), to_f64(K), to_f64(V)
    Oref, denref = ro.forward(Qd, Kd, Vd, list(W), w.sharpening, w.L, w.P, True)
    if n_prefill:
        for b in range(w.B):
            for h in range(w.H):
                A, Bs = ro.bucket_statistics(Kd[b, h, :n_prefill], Vd[b, h, :n_prefill], W[h], w.sharpening, w.L, w.P)
                ref = np.concatenate([Bs, A[:, :, None]], axis=2)
                got = to_f64(state[b, h])
                assert np.abs(got - ref).max() <= TOL[w.dtype] * np.abs(ref).max()
    else:
        assert float(state.abs().max()) == 0.0
    worst_o = worst_d = 0.0
    for t in range(n_prefill, n_prefill + n_steps):
        o, den = ra.race_attn_step(dp, Q[:, :, t].contiguous(), K[:, :, t].contiguous(), V[:, :, t].contiguous(),
                                   seeds, state)
        torch.cuda.synchronize()
        worst_o = max(worst_o, float(np.abs(to_f64(o) - Oref[:, :, t]).max() / np.abs(Oref[:, :, t]).max()))
        worst_d = max(worst_d, float(np.abs(to_f64(den) - denref[:, :, t]).max() / np.abs(denref[:, :, t]).max()))
    print("%s: prefill %d steps %d: O %.2e den %.2e" % (w.name, n_prefill, n_steps, worst_o, worst_d), flush=True)
    assert worst_o < TOL[w.dtype] and worst_d < TOL[w.dtype]


def test_decode_from_empty_state_fp32():
    _decode_against_oracle(Workload("dec-f32", 2, 2, 0, 64, 4, 4, 8.0, True, "f32"), 0, 24)


def test_decode_after_prefill_generic_family_fp32():
    _decode_against_oracle(Workload("dec-f32-prefill", 1, 2, 0, 64, 4, 4, 8.0, True, "f32", chunk=64), 150, 12)


def test_decode_after_prefill_mfma_family_bf16():
    w = Workload("dec-bf16-prefill", 1, 2, 0, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True, chunk=256)
    assert ra.race_attn_kernel_family(desc_of(Workload("x", 1, 2, 600, 128, 8, 6, 8.0, True, "bf16"))) == 2
    _decode_against_oracle(w, 600, 10)


def test_decode_from_empty_state_bf16_headline_shape():
    _decode_against_oracle(Workload("dec-bf16", 1, 4, 0, 128, 8, 6, 8.0, True, "bf16"), 0, 16)


@pytest.mark.parametrize("d,L,P", [(192, 3, 5), (256, 5, 2), (72, 17, 3), (64, 20, 8)])
def test_decode_odd_shapes_fp32(d, L, P):
    # column slots of 64..256 threads, more tables than slots, a slot count that does not divide the workgroup
    _decode_against_oracle(Workload("dec-odd-d%d-L%d-P%d" % (d, L, P), 1, 2, 0, d, L, P, 4.0, True, "f32"), 0, 6)


def test_later_steps_may_reuse_the_projection_in_the_workspace():
    w = Workload("dec-reuse", 2, 2, 10, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True)
    Q, K, V, _ = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    d = desc_of(w)
    d0 = ra.make_desc(w.B, w.H, 0, w.d, w.L, w.P, w.sharpening, True, d.dtype, 0)
    ws = torch.empty(ra.race_attn_step_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    runs = []
    for reuse in (False, True):
        state = ra.race_attn_state_init(d0, None, None, seeds)
        outs = []
        for t in range(w.N):
            s = None if (reuse and t > 0) else seeds
            o, den = ra.race_attn_step(d, Q[:, :, t].contiguous(), K[:, :, t].contiguous(), V[:, :, t].contiguous(), s,
                                       state, workspace=ws)
            outs += [o.clone(), den.clone()]
        torch.cuda.synchronize()
        runs.append(outs + [state])
    for a, b in zip(*runs):
        assert torch.equal(a, b)
