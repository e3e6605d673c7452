"""GPU parity on seeded random problem shapes: both kernel families, every compiled MFMA shape through padded
execution, causal and not, ragged lengths and odd segment lengths.  Each case is one check_case call (forward and
backward against the fp64 oracle, element by element)."""
import random

import pytest

import paper_2510_04008_amd as ra
from paper_2510_04008_amd.synth import Workload

from parity_util import check_case, desc_of

pytestmark = pytest.mark.gpu


def _cases():
    rng = random.Random(20251004)
    out = []
    for i in range(18):
        dtype = "bf16" if i % 3 else "f32"
        if dtype == "bf16":
            d = rng.choice([64, 128])
            P = rng.randint(1, 6)
            L = rng.randint(1, 16 if P <= 4 else 8)
        else:
            d = rng.choice([8, 24, 64, 96])
            P = rng.randint(1, 5)
            L = rng.randint(1, 6)
        B, H = rng.randint(1, 2), rng.randint(1, 3)
        N = rng.choice([3, 7, 33, 64, 95, 257, 600, 1111])    # (N = 1: dQ = dK = 0 exactly, covered with a floor elsewhere)
        causal = bool(rng.getrandbits(1))
        chunk = rng.choice([0, 32, 96, 160, 512]) if dtype == "bf16" else rng.choice([0, 8, 40, 64])
        beta = rng.choice([1.0, 2.0, 4.0])
        out.append(Workload("seeded-%02d-%s-d%d-P%d-L%d-N%d-%s-c%d" % (i, dtype, d, P, L, N, "c" if causal else "n", chunk),
                            B, H, N, d, L, P, beta, causal, dtype, normalize_qk=True, chunk=chunk))
    return out


@pytest.mark.parametrize("w", _cases(), ids=lambda w: w.name)
def test_seeded_shape(w):
    fam = ra.race_attn_kernel_family(desc_of(w))
    assert fam == (2 if w.dtype == "bf16" else 1)
    check_case(w)
