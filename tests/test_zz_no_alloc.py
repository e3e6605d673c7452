"""GPU test of race_attn_fwd_static, the forward pass for callers that cannot allocate: its kernels run on an
array inside the library instead of a caller's workspace.  Compared with race_attn_fwd on the same inputs, on two
calls in a row, the second on a smaller problem (the array keeps the first call's contents)."""
import pytest
import torch

import paper_2510_04008_amd as ra
from paper_2510_04008_amd import synth
from paper_2510_04008_amd.synth import Workload

from parity_util import TOL, desc_of

pytestmark = pytest.mark.gpu


def _both(w):
    Q, K, V, _ = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    d = desc_of(w)
    O_ref, den_ref = ra.race_attn_fwd(d, Q, K, V, seeds)          # also leaves the pinned image of W in the host cache
    O = torch.full_like(V, float("nan"))
    den = torch.full((w.B, w.H, w.N), float("nan"), dtype=torch.float32, device="cuda")
    ra.race_attn_fwd_static(d, Q, K, V, seeds, O, den)
    torch.cuda.synchronize()
    return O, den, O_ref, den_ref


def _close(a, b, tol):
    a, b = a.double(), b.double()
    assert torch.isfinite(a).all()
    return ((a - b).abs().max() / b.abs().max()).item() < tol


@pytest.mark.parametrize("family_case", ["mfma", "generic"])
def test_two_calls_in_a_row_the_second_smaller(family_case):
    if family_case == "mfma":
        big = Workload("static-big", 1, 4, 5000, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True, chunk=512)
        small = Workload("static-small", 1, 2, 700, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True, chunk=256)
    else:
        big = Workload("static-big-f32", 1, 2, 1024, 64, 4, 4, 8.0, False, "f32")
        small = Workload("static-small-f32", 1, 1, 300, 64, 4, 4, 8.0, True, "f32", chunk=64)
    for w in (big, small):
        O, den, O_ref, den_ref = _both(w)
        # same plan, same kernels, same order of every sum: bit-identical
        assert torch.equal(O, O_ref) and torch.equal(den, den_ref), w.name


def test_a_problem_beyond_the_array_runs_on_longer_segments():
    # the default plan wants 32 segments x 4 heads x 258 KiB = 33.8 MB of statistics next to 12.6 MB of hashed rows; the
    # entry point doubles the segment length until everything fits its 32 MiB, which changes the order of the sums over
    # segments and nothing else
    w = Workload("static-replanned", 1, 4, 8192, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True, chunk=256)
    assert ra.race_attn_workspace_bytes(desc_of(w)) > (32 << 20)
    O, den, O_ref, den_ref = _both(w)
    assert _close(O, O_ref, TOL["bf16"]) and _close(den, den_ref, TOL["bf16"])
    # and a smaller call right after it
    w2 = Workload("static-after", 1, 1, 100, 128, 8, 6, 8.0, False, "bf16", normalize_qk=True)
    O, den, O_ref, den_ref = _both(w2)
    assert torch.equal(O, O_ref) and torch.equal(den, den_ref)


def test_unprepared_seeds_are_refused():
    w = Workload("static-cold", 1, 2, 256, 128, 8, 6, 8.0, True, "bf16")
    Q, K, V, _ = synth.make_inputs(w, "cuda")
    O = torch.zeros_like(V)
    den = torch.zeros((1, 2, 256), dtype=torch.float32, device="cuda")
    with pytest.raises(ra.RaceAttnError) as e:
        ra.race_attn_fwd_static(desc_of(w), Q, K, V, [0x5EED0001, 0x5EED0002], O, den)
    assert e.value.status == ra.RACE_ERR_NOT_READY
    torch.cuda.synchronize()
    assert O.abs().max().item() == 0.0          # nothing was launched
