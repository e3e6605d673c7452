"""GPU parity of problems served by a larger compiled shape of the bf16 MFMA family (padding tables are empty,
padding hyperplanes put all their mass on one side), against the fp64 oracle and through the C ABI: the paper's own
scaling grid (P, L) in {(2,2), (3,3), (4,4)} at d = 128 and an odd shape at d = 64."""
import numpy as np
import pytest
import torch

import paper_2510_04008_amd as ra
from oracle import race_oracle as ro
from paper_2510_04008_amd import synth
from paper_2510_04008_amd.synth import Workload

from parity_util import TOL, check_case, check_dbeta, desc_of, oracle_w, to_f64

pytestmark = pytest.mark.gpu

GRID = [(2, 2, 128), (3, 3, 128), (4, 4, 128), (3, 5, 64), (1, 1, 128), (4, 16, 128),
        # beyond four hyperplanes: the padded instantiations of the L = 8, P = 6 shape
        (5, 5, 128), (6, 4, 128), (5, 8, 128), (6, 8, 64), (5, 3, 64),
        # the 64- and 128-row shapes (two and four wavefronts carry the statistics in the gradient kernels)
        (4, 3, 128), (4, 8, 128), (3, 7, 128), (4, 5, 128)]


@pytest.mark.parametrize("P,L,d", GRID)
@pytest.mark.parametrize("causal", [True, False])
def test_padded_shapes_forward_backward(P, L, d, causal):
    w = Workload("pad-P%d-L%d-d%d-%s" % (P, L, d, "c" if causal else "n"), 1, 2, 777, d, L, P, 4.0, causal, "bf16",
                 normalize_qk=True, chunk=256)
    assert ra.race_attn_kernel_family(desc_of(w)) == 2
    check_case(w)


def test_padded_shape_raw_inputs_and_batch():
    # raw N(0,1) rows (|z| ~ 11: saturated tanh).  At beta = 8 and only 4 x 16 buckets the first few causal tokens
    # have Den ~ 1e-9 (query and the handful of keys before it share no bucket); every token is compared
    w = Workload("pad-raw", 2, 3, 1000, 128, 4, 4, 8.0, True, "bf16", chunk=128)
    assert ra.race_attn_kernel_family(desc_of(w)) == 2
    check_case(w)
    check_case(Workload("pad-raw-beta2", 2, 3, 1000, 128, 4, 4, 2.0, True, "bf16", chunk=128))


def test_padded_shape_taps_report_the_problems_own_corners():
    w = Workload("pad-taps", 1, 2, 500, 128, 3, 3, 4.0, True, "bf16", normalize_qk=True)
    Q, K, V, _ = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    d = desc_of(w)
    codes, phi = ra.race_attn_debug_hash(d, Q, seeds, want_phi=True)
    A, Bsum = ra.race_attn_debug_buckets(d, K, V, seeds)
    torch.cuda.synchronize()
    assert tuple(codes.shape) == (1, 2, 500, 3) and tuple(phi.shape) == (1, 2, 500, 3, 8)
    W = oracle_w(w, seeds)
    Qh, Kh, Vh = to_f64(Q), to_f64(K), to_f64(V)
    for h in range(w.H):
        z = ro.project(Qh[0, h], W[h], w.L, w.P)
        ref = ro.hard_codes(Qh[0, h], W[h], w.L, w.P)
        got = codes[0, h].cpu().numpy().astype(np.int64)
        tau = 2.0 ** -16 * np.linalg.norm(Qh[0, h], axis=1)[:, None, None] * np.linalg.norm(W[h], axis=1).reshape(1, w.L, w.P)
        band = (np.abs(z) <= tau).any(axis=2)
        assert int(((got != ref) & ~band).sum()) == 0 and got.max() < 8
        ref_phi = ro.soft_hash(Qh[0, h], W[h], w.sharpening, w.L, w.P)
        assert np.abs(to_f64(phi[0, h]) - ref_phi).max() < 2.0 ** -8
        Ar, Br = ro.bucket_statistics(Kh[0, h], Vh[0, h], W[h], w.sharpening, w.L, w.P)
        assert np.abs(to_f64(A[0, h]) - Ar).max() <= TOL["bf16"] * np.abs(Ar).max()
        assert np.abs(to_f64(Bsum[0, h]) - Br).max() <= TOL["bf16"] * np.abs(Br).max()


def test_padded_shape_beta_cotangent_and_decode_prefill():
    # a mild temperature: the terms do not cancel much and the tensors' measure applies
    check_dbeta(Workload("pad-beta-mild", 1, 2, 900, 128, 4, 4, 1.0, True, "bf16", normalize_qk=True, chunk=256))
    check_dbeta(Workload("pad-beta", 1, 2, 900, 128, 4, 4, 4.0, True, "bf16", normalize_qk=True, chunk=256))
    check_dbeta(Workload("pad-beta-33", 1, 2, 900, 128, 3, 3, 4.0, False, "bf16", normalize_qk=True))
    # the decoding state of a padded problem has the problem's own shape
    w = Workload("pad-state", 1, 2, 600, 128, 3, 3, 4.0, True, "bf16", normalize_qk=True)
    _, K, V, _ = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    state = ra.race_attn_state_init(desc_of(w), K, V, seeds)
    torch.cuda.synchronize()
    assert tuple(state.shape) == (1, 2, 3, 8, 129)
    W = oracle_w(w, seeds)
    for h in range(w.H):
        Ar, Br = ro.bucket_statistics(to_f64(K)[0, h], to_f64(V)[0, h], W[h], w.sharpening, w.L, w.P)
        ref = np.concatenate([Br, Ar[:, :, None]], axis=2)
        assert np.abs(to_f64(state[0, h]) - ref).max() <= TOL["bf16"] * np.abs(ref).max()
