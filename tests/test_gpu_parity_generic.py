"""GPU parity of the generic (fp32-arithmetic) kernel family against the fp64 oracle, through the C ABI."""
import os

import numpy as np
import pytest
import torch

import paper_2510_04008_amd as ra
from oracle import race_oracle as ro
from paper_2510_04008_amd import synth
from paper_2510_04008_amd.synth import Workload

from parity_util import TOL, check_case, desc_of, oracle_w, rel_err, run_gpu, to_f64

pytestmark = pytest.mark.gpu


def test_config1_tiny_noncausal_fp32():
    g, r, errs = check_case(synth.C1)
    assert ra.race_attn_kernel_family(desc_of(synth.C1)) == 1


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_multi_segment(causal, dtype, monkeypatch):
    # several segments, a short last segment, a short last tile, several heads and batches
    monkeypatch.setenv("RACE_ATTN_FORCE_GENERIC", "1")
    w = Workload("ragged", 2, 3, 1003, 32, 3, 3, 2.0, causal, dtype, normalize_qk=True, chunk=96)
    check_case(w)


@pytest.mark.parametrize("N", [1, 5, 8, 9])
def test_tiny_sequences(N):
    # a single token attends only to itself: O = V and dQ = dK = 0 exactly, so those two are
    # compared on an absolute scale
    floors = {"dQ": 1.0, "dK": 1.0} if N == 1 else None
    check_case(Workload("tinyN%d" % N, 1, 2, N, 16, 2, 2, 1.5, True, "f32", normalize_qk=True), floors=floors)
    check_case(Workload("tinyN%d-nc" % N, 1, 2, N, 16, 2, 2, 1.5, False, "f32", normalize_qk=True), floors=floors)


@pytest.mark.parametrize("L,P,d", [(1, 1, 8), (2, 8, 64), (5, 2, 256), (8, 6, 128)])
def test_shape_extremes(L, P, d):
    check_case(Workload("shape", 1, 2, 300, d, L, P, 3.0, True, "f32", normalize_qk=True))


def test_saturated_regime_raw_gaussian_inputs():
    # rows of norm ~ sqrt(d): |z| ~ 8, tanh saturates, phi is almost one-hot
    check_case(Workload("saturated", 1, 2, 777, 64, 4, 4, 8.0, True, "f32", chunk=128))


def test_headline_shape_bf16_generic_family(monkeypatch):
    monkeypatch.setenv("RACE_ATTN_FORCE_GENERIC", "1")
    check_case(Workload("headline-small", 1, 4, 2048, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True, chunk=512))


def test_hash_tap_codes_and_phi():
    w = Workload("hash", 1, 2, 513, 64, 4, 4, 8.0, False, "f32", normalize_qk=True)
    Q, K, V, dO = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    codes, phi = ra.race_attn_debug_hash(desc_of(w), K, seeds, want_phi=True)
    torch.cuda.synchronize()
    W = oracle_w(w, seeds)
    Kh = to_f64(K)
    mism_out_of_band = 0
    in_band = 0
    for h in range(w.H):
        z = ro.project(Kh[0, h], W[h], w.L, w.P)
        ref_codes = ro.hard_codes(Kh[0, h], W[h], w.L, w.P)
        # a sign may differ from the fp64 oracle only where |z| is inside the fp32 rounding band
        tau = 2.0 ** -16 * np.linalg.norm(Kh[0, h], axis=1)[:, None, None] * \
            np.linalg.norm(W[h], axis=1).reshape(1, w.L, w.P)
        band = (np.abs(z) <= tau).any(axis=2)
        got = codes[0, h].cpu().numpy().astype(np.int64)
        in_band += int(band.sum())
        mism_out_of_band += int(((got != ref_codes) & ~band).sum())
        ref_phi = ro.soft_hash(Kh[0, h], W[h], w.sharpening, w.L, w.P)
        assert np.abs(phi[0, h].cpu().numpy() - ref_phi).max() < 1e-5
    print("hash tap: in-band projections", in_band, "out-of-band mismatches", mism_out_of_band, flush=True)
    assert mism_out_of_band == 0


def test_bucket_tap():
    w = Workload("buckets", 2, 2, 700, 32, 3, 3, 4.0, True, "f32", normalize_qk=True, chunk=128)
    Q, K, V, dO = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    A, Bsum = ra.race_attn_debug_buckets(desc_of(w), K, V, seeds)
    torch.cuda.synchronize()
    W = oracle_w(w, seeds)
    for b in range(w.B):
        for h in range(w.H):
            rA, rB = ro.bucket_statistics(to_f64(K)[b, h], to_f64(V)[b, h], W[h], w.sharpening, w.L, w.P)
            assert rel_err(A[b, h], rA) < 1e-5 and rel_err(Bsum[b, h], rB) < 1e-5


def test_constant_values_and_determinism():
    w = Workload("ones", 1, 2, 640, 32, 4, 3, 4.0, True, "f32", normalize_qk=True, chunk=128)
    Q, K, V, dO = synth.make_inputs(w, "cuda")
    V1 = torch.full_like(V, 1.0)
    g1 = run_gpu(w, (Q, K, V1, dO))
    assert (g1["O"] - 1.0).abs().max().item() < 1e-5          # rows of the attention matrix sum to one
    assert g1["dQ"].abs().max().item() < 1e-4 and g1["dK"].abs().max().item() < 1e-4
    g2 = run_gpu(w, (Q, K, V, dO))
    g3 = run_gpu(w, (Q, K, V, dO))
    for n in ("O", "den", "dQ", "dK", "dV"):
        assert torch.equal(g2[n], g3[n]), n                    # bit-identical from run to run
    # total value gradient = total upstream gradient
    assert torch.allclose(g2["dV"].sum(dim=2), dO.sum(dim=2), atol=2e-3)


def test_causal_outputs_ignore_the_future():
    w = Workload("leak", 1, 1, 512, 32, 4, 3, 4.0, True, "f32", normalize_qk=True, chunk=128)
    Q, K, V, dO = synth.make_inputs(w, "cuda")
    V2 = V.clone()
    V2[:, :, :300] = 0
    g = run_gpu(w, (Q, K, V2, dO))
    assert g["O"][:, :, :300].abs().max().item() == 0.0        # values before token 300 are all zero
    assert g["O"][:, :, 300:].abs().max().item() > 0


def test_empty_sequence_and_error_reporting():
    d = ra.make_desc(1, 1, 0, 16, 2, 2, 1.0, True, ra.RACE_F32)
    e = torch.empty((1, 1, 0, 16), device="cuda")
    O, den = ra.race_attn_fwd(d, e, e, e, [1])
    assert O.numel() == 0
    d = ra.make_desc(1, 1, 64, 16, 2, 2, 1.0, True, ra.RACE_F32)
    x = torch.zeros((1, 1, 64, 16), device="cuda")
    with pytest.raises(ra.RaceAttnError):
        ra.race_attn_fwd(d, x, x, x, [1], workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))


@pytest.mark.gpu
def test_calibration_copy_copies():
    import torch
    src = torch.randint(0, 255, (3 * 1024 * 1024 + 16,), dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros_like(src)
    ra.race_attn_calibration_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


def test_beta_cotangent_fp32():
    from parity_util import check_dbeta
    check_dbeta(synth.C1)
    check_dbeta(Workload("g-beta-causal", 2, 2, 300, 32, 3, 3, 2.0, True, "f32", chunk=64))


def test_beta_cotangent_bf16_generic_shape(monkeypatch):
    from parity_util import check_dbeta
    monkeypatch.setenv("RACE_ATTN_FORCE_GENERIC", "1")
    check_dbeta(Workload("g-beta-bf16", 1, 2, 500, 64, 4, 3, 4.0, True, "bf16", chunk=128))


def test_calibration_mfma_runs_and_fills_the_sink():
    sink = torch.full((16 * 256,), float("nan"), dtype=torch.float32, device="cuda:0")
    flop = ra.race_attn_calibration_mfma(16, 8, sink)
    torch.cuda.synchronize()
    assert flop == 16 * 4 * 8 * 4 * 32768
    assert torch.isfinite(sink).all() and (sink > 0).all()
    for nv in (4, 8, 16):       # the variants with vector multiplies between the matrix instructions
        sink.fill_(float("nan"))
        ra.race_attn_calibration_mfma(16, 8, sink, vector_ops=nv)
        torch.cuda.synchronize()
        assert torch.isfinite(sink).all() and (sink > 0).all()
