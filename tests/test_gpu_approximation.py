"""Approximation-quality harness: the HIP path against the attention it estimates (P-powered angular kernel,
Theorem 1), on synthetic unit-norm queries and keys, as a function of the number of tables L and the temperature.

Two statements per (L, beta): the kernels reproduce the oracle's RACE output within the parity tolerance, and so
their distance to the target is the oracle's; and the distances follow the theorem's two terms (variance ~ L^-1/2
at a high temperature, bias falling with beta at many tables).  Prints the table that the design notes quote.
"""
import math

import numpy as np
import pytest
import torch

import paper_2510_04008_amd as ra
from oracle import angular
from oracle import race_oracle as ro
from paper_2510_04008_amd import synth
from paper_2510_04008_amd.synth import Workload

from parity_util import TOL, desc_of, oracle_w, rel_err, to_f64

pytestmark = pytest.mark.gpu


def _clustered(gen, N, d, centres=8, spread=0.35):
    """Unit-norm queries and keys scattered around shared directions, and values that say which direction a key
    belongs to (plus noise): attention rows are far from uniform and the output depends on how sharp they are."""
    c = torch.randn(centres, d, generator=gen, dtype=torch.float64)
    c /= c.norm(dim=1, keepdim=True)
    cv = torch.randn(centres, d, generator=gen, dtype=torch.float64)
    def rows(pick):
        x = c[pick] + spread / math.sqrt(d) * torch.randn(N, d, generator=gen, dtype=torch.float64)
        return x / x.norm(dim=1, keepdim=True)
    pq, pk = torch.randint(0, centres, (N,), generator=gen), torch.randint(0, centres, (N,), generator=gen)
    V = cv[pk] + 0.1 * torch.randn(N, d, generator=gen, dtype=torch.float64)
    return rows(pq), rows(pk), V


def test_distance_to_angular_attention_by_tables_and_temperature():
    # every head gets the same Q, K, V and its own W: the heads are independent draws of the estimator, and the
    # mean of their outputs behaves like H times as many tables (its error is mostly the bias of the softening)
    B, H, N, d, P = 1, 16, 1024, 128, 4
    gen = torch.Generator().manual_seed(20)
    Q, K, V = (t.to(torch.bfloat16).expand(B, H, N, d).contiguous().cuda() for t in _clustered(gen, N, d))
    Qh, Kh, Vh = to_f64(Q)[0, 0], to_f64(K)[0, 0], to_f64(V)[0, 0]
    target = angular.angular_attention(Qh, Kh, Vh, P)
    rows, per_head, pooled = [], {}, {}
    for L in (2, 4, 8, 16):
        for beta in (1.0, 4.0, 16.0, 64.0):
            w = Workload("approx", B, H, N, d, L, P, beta, False, "bf16")
            assert ra.race_attn_kernel_family(desc_of(w)) == 2
            seeds = synth.projection_seeds(w)
            W = oracle_w(w, seeds)
            O, _ = ra.race_attn_fwd(desc_of(w), Q, K, V, seeds)
            torch.cuda.synchronize()
            Og = to_f64(O)[0]
            ref = np.stack([ro.forward_linear(Qh, Kh, Vh, W[h], beta, L, P)[0] for h in range(H)])
            assert rel_err(O[0], ref) < TOL["bf16"]
            e_gpu = float(np.mean([angular.rms_error(Og[h], target) for h in range(H)]))
            e_ref = float(np.mean([angular.rms_error(ref[h], target) for h in range(H)]))
            assert abs(e_gpu - e_ref) < 0.02 * e_ref + 2e-3
            per_head[(L, beta)] = e_gpu
            pooled[(L, beta)] = angular.rms_error(Og.mean(axis=0), target)
            rows.append("| %2d | %5.1f | %.4f | %.4f | %.4f | %.4f |" % (L, beta, e_gpu, e_ref, pooled[(L, beta)],
                                                                       angular.rms_error(ref.mean(axis=0), target)))
    scale = float(np.sqrt((target ** 2).sum(axis=1).mean()))
    print("\nrms error against angular attention (gamma = P = %d), N=%d d=%d, %d heads; rms |O_i| of the target = %.3f"
          % (P, N, d, H, scale))
    print("| L | beta | kernels, per head | oracle RACE, per head | kernels, mean of heads | oracle, mean of heads |")
    print("|---|---|---|---|---|---|")
    print("\n".join(rows), flush=True)
    # variance term: at a high temperature the per-head error falls with the number of tables, about like L^-1/2
    assert per_head[(2, 64.0)] > per_head[(4, 64.0)] > per_head[(8, 64.0)] > per_head[(16, 64.0)]
    assert 1.7 < per_head[(2, 64.0)] / per_head[(16, 64.0)] < 6.0          # sqrt(8) = 2.8
    # bias term: pooled over the heads (16 x 16 tables) the error falls as the temperature rises
    assert pooled[(16, 1.0)] > pooled[(16, 4.0)] > pooled[(16, 16.0)]
    assert pooled[(16, 1.0)] > 2 * pooled[(16, 64.0)]
