"""Seeded synthetic inputs for tests and benchmarks.  Holds none of the method's arithmetic: it only
draws tensors of the shapes and value distributions of the benchmark workloads.

The paper's scaling study runs one attention layer on tensors of a given shape (B=1, H=4, d=128),
no dataset involved, so i.i.d. Gaussian tensors are that workload itself.  Two regimes:
raw N(0,1) rows (norm ~ sqrt(d): projections are large, tanh saturates) and L2-normalised rows
(projections ~ N(0,1), the regime of the paper's analysis).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    L: int
    P: int
    sharpening: float
    causal: bool
    dtype: str            # "f32" or "bf16"
    normalize_qk: bool = False     # input recipe: rows of Q and K are generated with unit length
    chunk: int = 0
    unit_qk: bool = False          # descriptor option: the layer divides the rows of Q and K by their norms

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, N: int, name: str = None) -> "Workload":
        return Workload(name or ("%s@N=%d" % (self.name, N)), self.B, self.H, N, self.d, self.L, self.P,
                        self.sharpening, self.causal, self.dtype, self.normalize_qk, self.chunk, self.unit_qk)


# The five benchmark configurations.
C1 = Workload("C1-tiny-noncausal-f32", 1, 1, 1024, 64, 4, 4, 8.0, False, "f32")
C2 = Workload("C2-causal-bf16-64K", 1, 4, 65536, 128, 8, 6, 8.0, True, "bf16", normalize_qk=True, chunk=1024)
C3 = Workload("C3-noncausal-bf16-16K", 8, 8, 16384, 64, 16, 4, 4.0, False, "bf16")
C4 = Workload("C4-causal-bf16-4M", 1, 4, 4194304, 128, 8, 6, 8.0, True, "bf16")
C5 = Workload("C5-causal-bf16-12M", 1, 4, 12582912, 128, 8, 6, 8.0, True, "bf16")
# the paper's own scaling grid (Section 4, single-layer stress test): (P, L) in {(2,2), (3,3), (4,4)}, B=1, H=4, d=128
G22 = Workload("G22-causal-bf16-1M", 1, 4, 1048576, 128, 2, 2, 8.0, True, "bf16")
G33 = Workload("G33-causal-bf16-1M", 1, 4, 1048576, 128, 3, 3, 8.0, True, "bf16")
G44 = Workload("G44-causal-bf16-1M", 1, 4, 1048576, 128, 4, 4, 8.0, True, "bf16")
WORKLOADS = {w.name.split("-")[0]: w for w in (C1, C2, C3, C4, C5, G22, G33, G44)}

SEED_QKV, SEED_W, SEED_DO = 0, 1, 2
_SLICE = 1 << 18      # tokens generated at a time (bounds the fp32 temporary)


def projection_seeds(w: Workload, base: int = SEED_W):
    """One 64-bit seed per head."""
    return [base + 1000003 * h for h in range(w.H)]


def _fill(out: torch.Tensor, gen: torch.Generator, normalize: bool):
    B, H, N, d = out.shape
    for n0 in range(0, N, _SLICE):
        n1 = min(N, n0 + _SLICE)
        x = torch.randn((B, H, n1 - n0, d), generator=gen, dtype=torch.float32, device=gen.device)
        if normalize:
            x = x / x.norm(dim=-1, keepdim=True)
        out[:, :, n0:n1] = x.to(out.dtype).to(out.device)
    return out


def make_inputs(w: Workload, device="cuda", on_device_rng: bool = False
                ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """Q, K, V, dO as (B, H, N, d) tensors of the workload's element type on `device`.

    With on_device_rng the values come from the device's generator (large benchmark tensors; the same
    buffers are what the oracle reads back, so parity does not depend on the generator).  Otherwise
    they come from the CPU generator and are identical on every machine.
    """
    gdev = device if on_device_rng else "cpu"
    tensors = []
    for i, (seed, norm) in enumerate(((SEED_QKV, w.normalize_qk), (SEED_QKV, w.normalize_qk),
                                      (SEED_QKV, False), (SEED_DO, False))):
        gen = torch.Generator(device=gdev)
        gen.manual_seed(seed * 7919 + i)
        t = torch.empty((w.B, w.H, w.N, w.d), dtype=w.torch_dtype, device=device)
        tensors.append(_fill(t, gen, norm))
    return tuple(tensors)
