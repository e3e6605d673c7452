"""Host-side logic of bench.py (no GPU): the per-kernel credit table adds up to the algorithmic counts, the committed
HBM-traffic summary belongs to the committed kernel sources, and a run on more than one GPU is refused."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench                                     # noqa: E402
from paper_2510_04008_amd import synth           # noqa: E402

MFMA_KERNELS = ("hash_rows", "stream_totals_kv", "segment_scan", "stream_forward", "stream_totals_qg", "stream_grad_v",
                "grad_q", "grad_k")


def test_kernel_credits_add_up_to_the_algorithmic_counts():
    # forward Proj + 2U, backward 2 Proj + 4U; every tensor of the problem statement moved once per pass
    for w in (synth.C2, synth.C3, synth.C5, synth.G44):
        proj, U, nbytes = bench.algorithmic_counts(w)
        R = 1 << w.P
        assert proj == 4 * w.d * w.L * w.P and U == 2 * w.L * R * (w.d + 1) and nbytes == 12 * w.d * 2 + 8
        shares = bench.kernel_shares(w)
        assert sum(shares[k][0] for k in MFMA_KERNELS) == 3 * proj + 6 * U
        assert sum(shares[k][1] for k in MFMA_KERNELS) == nbytes
        # the kernels that exist only because the sequence is cut into segments get nothing
        assert shares["stream_totals_kv"] == shares["stream_totals_qg"] == shares["segment_scan"] == (0.0, 0.0)


def test_headline_counts_are_the_published_ones():
    proj, U, nbytes = bench.algorithmic_counts(synth.C5)
    assert (proj, U, nbytes) == (24576, 132096, 3080) and 3 * proj + 6 * U == 866304


def test_committed_traffic_summary_was_measured_on_the_committed_sources():
    table, source = bench.measured_traffic(synth.C5)
    assert table is not None, source               # a stale summary: re-run the two counter passes it names
    assert source == os.path.join("profiles", "hbm_traffic_c5_pmc.md")
    assert set(MFMA_KERNELS) <= set(table)
    # more than the algorithmic bytes (operands are read again by later passes), less than three times as much
    step = sum(table[k] * (2 if k == "segment_scan" else 1) for k in MFMA_KERNELS)
    assert 3080 < step < 3 * 3080
    # a workload without a summary says so instead of borrowing another workload's figures
    table, reason = bench.measured_traffic(synth.C3)
    assert table is None and "no counter summary" in reason


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
