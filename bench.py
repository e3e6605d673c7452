#!/usr/bin/env python3
"""Benchmark: RACE Attention forward+backward tokens/s on one MI355X, with the dominant kernel's
roofline fraction and the fp64 oracle timed on the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5|C4|C2|C3] [--tokens N]

A step is one race_attn_fwd plus one backward pass (race_attn_bwd_saved on the forward's workspace, or
race_attn_bwd with --bwd-recompute) over one batch of synthetic, seeded inputs that are resident in HBM
before the timed region starts.  Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_BF16_FLOPS = 2.5e15
PEAK_FP32_VECTOR_FLOPS = 157.3e12      # the generic kernel family computes on the vector ALUs in fp32
PEAK_HBM_BYTES = 8.0e12


def algorithmic_counts(w):
    """Per token-head work the method itself needs (no N x N work, no implementation extras):
    Proj = 4 d L P (projections of Q and K), U = 2 L R (d+1) (one contraction with the bucket
    statistics).  forward = Proj + 2U, backward = 2 Proj + 4U, bytes = 12 d s + 8."""
    R = 1 << w.P
    proj = 4 * w.d * w.L * w.P
    U = 2 * w.L * R * (w.d + 1)
    s = 2 if w.dtype == "bf16" else 4
    return proj, U, 12 * w.d * s + 8


def kernel_shares(w):
    """Algorithmic work per token-head credited to each kernel, (flops, HBM bytes); the flops add up to 3 Proj + 6 U and
    the bytes to 12 d s + 8.  The segment-total and scan kernels exist only because the sequence is cut into segments
    and get 0.  Bytes: every tensor of the problem statement is credited once per pass, to the kernel that first
    needs it (forward: Q, K to the hashing kernel, V, O, den to the streaming pass; backward: dO, O, den, dV to the
    dV pass, Q, dQ to the dQ pass, K, V, dK to the dK pass)."""
    proj, U, _ = algorithmic_counts(w)
    s = 2 if w.dtype == "bf16" else 4
    ds = w.d * s
    return {
        "hash_rows": (proj, 2 * ds),                 # projections of Q and K
        "stream_forward": (2 * U, 2 * ds + 4),       # accumulate, read-out
        "stream_grad_v": (2 * U, 3 * ds + 4),        # cotangent statistics, dV read-out
        "grad_q": (U + proj, 2 * ds),                # dphi_Q, projection of Q again (tanh and its derivative), dQ = dz . W
        "grad_k": (U + proj, 3 * ds),                # dphi_K, same
        "stream_totals_kv": (0.0, 0.0), "stream_totals_qg": (0.0, 0.0), "segment_scan": (0.0, 0.0),
        # generic family: one replay kernel forward; the key/value kernel forms dV and dK
        "simple_fwd_replay": (proj + 2 * U, 4 * ds + 4),
        "simple_bwd_keyvalue": (proj + 2 * U + U + proj / 2, 6 * ds + 4),
        "simple_bwd_query": (U + proj / 2, 2 * ds),
    }


def source_hash() -> str:
    """SHA-256 over the library's sources: what a stored counter measurement is valid for."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2510_04008_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def measured_traffic(w):
    """HBM bytes per token-head and launch, per kernel, from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a plain copy of known size), or
    (None, reason): the summary names the sources it was measured on, and a summary of other sources is not used."""
    import re
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s_pmc.md" % w.name.split("-")[0].lower())
    if not os.path.exists(path):
        return None, "no counter summary for this workload under profiles/"
    text = open(path).read()
    m = re.search(r"source-sha256:\s*([0-9a-f]{64})", text)
    t = re.search(r"bytes-per-token-head:\s*(.+)", text)
    if not m or not t:
        return None, "%s holds no machine-readable table" % os.path.relpath(path, ROOT)
    if m.group(1) != source_hash():
        return None, "%s was measured on other kernel sources (re-run the two --pmc passes it names)" % os.path.relpath(path, ROOT)
    table = {k: float(v) for k, v in (kv.split("=") for kv in t.group(1).split())}
    return table, os.path.relpath(path, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--print-source-hash", action="store_true", help="print the hash a counter summary must carry, and exit")
    ap.add_argument("--workload", default="C5")
    ap.add_argument("--tokens", type=int, default=0, help="override N of the workload")
    ap.add_argument("--chunk", type=int, default=-1, help="override the scan segment length in tokens (0 = let the library choose)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=196608)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--bwd-recompute", action="store_true",
                    help="time race_attn_bwd (derives the key/value statistics again) instead of race_attn_bwd_saved")
    ap.add_argument("--unit-qk", action="store_true",
                    help="descriptor option unit_qk: the layer divides the rows of Q and K by their norms (not the headline workload)")
    ap.add_argument("--noncausal", action="store_true", help="run the workload's shape without the causal mask (Algorithm 1)")
    ap.add_argument("--forward-only", action="store_true", help="time race_attn_fwd alone (inference; not the headline metric)")
    ap.add_argument("--sharpening", type=float, default=None, help="override the temperature (inf = hard hash, forward only)")
    ap.add_argument("--no-attainable", action="store_true", help="skip the copy / MFMA-loop calibration launches")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the warm-up, run one plain copy kernel of this many MiB (scale for byte counters)")
    args = ap.parse_args()
    if args.print_source_hash:
        print(source_hash())
        return 0
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on one GPU; --gpus %d is not supported "
                         "(the path has no collectives: a sequence would shard by batch and heads, or along N with the bucket "
                         "statistics exchanged once per segment scan)\n" % args.gpus)
        return 2

    import numpy as np
    import torch
    import paper_2510_04008_amd as ra
    from paper_2510_04008_amd import synth

    w = synth.WORKLOADS[args.workload]
    if args.tokens:
        w = w.scaled(args.tokens)
    if args.chunk >= 0:
        w = dataclasses.replace(w, chunk=args.chunk)
    if args.unit_qk:
        w = dataclasses.replace(w, name=w.name + "+unit_qk", unit_qk=True)
    if args.noncausal:
        w = dataclasses.replace(w, name=w.name.replace("causal", "noncausal"), causal=False)
    if args.sharpening is not None:
        w = dataclasses.replace(w, name=w.name + "+beta=%g" % args.sharpening, sharpening=args.sharpening)
        if args.sharpening == float("inf"):
            args.forward_only = True
    dev = "cuda:0"
    torch.cuda.set_device(0)
    desc = ra.make_desc(w.B, w.H, w.N, w.d, w.L, w.P, w.sharpening, w.causal,
                        ra.RACE_F32 if w.dtype == "f32" else ra.RACE_BF16, w.chunk, w.unit_qk)
    family = ra.race_attn_kernel_family(desc)
    if family == 0:
        raise SystemExit("unsupported workload")
    seeds = synth.projection_seeds(w)

    t_gen = time.perf_counter()
    Q, K, V, dO = synth.make_inputs(w, dev, on_device_rng=True)
    O = torch.empty_like(V)
    den = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=dev)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    ws = torch.empty(ra.race_attn_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    sys.stderr.write("inputs resident after %.1f s; workspace %.1f MiB; kernel family %d\n"
                     % (time.perf_counter() - t_gen, ws.numel() / 2 ** 20, family))

    # The backward pass of a training step follows the forward pass of the same inputs, whose workspace still
    # holds the key/value statistics at segment starts: race_attn_bwd_saved reads them (bit-identical results);
    # --bwd-recompute times race_attn_bwd, which derives them again from K and V.
    def step():
        ra.race_attn_fwd(desc, Q, K, V, seeds, O=O, den=den, workspace=ws)
        if args.forward_only:
            return
        if args.bwd_recompute:
            ra.race_attn_bwd(desc, Q, K, V, O, den, dO, seeds, dQ=dQ, dK=dK, dV=dV, workspace=ws)
        else:
            ra.race_attn_bwd_saved(desc, Q, K, V, O, den, dO, seeds, ws, dQ=dQ, dK=dK, dV=dV)

    if args.calibration_copy_mib:
        src = torch.randint(0, 256, (args.calibration_copy_mib << 20,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        ra.race_attn_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    attainable = None
    if not args.no_attainable:
        # what this machine reaches on a plain copy and on a dense MFMA loop, next to the published peaks
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 256)
        dst = torch.empty_like(src)
        sink = torch.empty(8192 * 256, dtype=torch.float32, device=dev)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(8)]
        ra.race_attn_calibration_copy(dst, src)
        ra.race_attn_calibration_mfma(8192, 64, sink)
        ev[0].record(); ra.race_attn_calibration_copy(dst, src); ev[1].record()
        ev[2].record(); flop = ra.race_attn_calibration_mfma(8192, 2048, sink); ev[3].record()
        # the same loop with 8 and 16 independent vector multiplies after every matrix instruction: what is left of the
        # matrix rate for a kernel that builds its operands with the vector ALU (these kernels issue 11-17 vector
        # instructions per matrix instruction)
        ev[4].record(); ra.race_attn_calibration_mfma(8192, 2048, sink, vector_ops=8); ev[5].record()
        ev[6].record(); ra.race_attn_calibration_mfma(8192, 2048, sink, vector_ops=16); ev[7].record()
        torch.cuda.synchronize()
        attainable = {"hbm_copy_GBps": 2 * src.numel() / (1e-3 * ev[0].elapsed_time(ev[1])) / 1e9,
                      "mfma_bf16_TFLOPs": flop / (1e-3 * ev[2].elapsed_time(ev[3])) / 1e12,
                      "mfma_bf16_TFLOPs_with_8_vector_ops_each": flop / (1e-3 * ev[4].elapsed_time(ev[5])) / 1e12,
                      "mfma_bf16_TFLOPs_with_16_vector_ops_each": flop / (1e-3 * ev[6].elapsed_time(ev[7])) / 1e12,
                      "note": "1 GiB copy kernel (read + write counted) and a register-operand "
                              "v_mfma_f32_32x32x16_bf16 loop (alone, and with 8 or 16 independent v_mul_f32 after every "
                              "matrix instruction), one launch each, HIP events"}
        del src, dst, sink

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ra.race_attn_profile_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = ra.race_attn_profile_read()
    ra.race_attn_profile_enable(False)

    # the step time is the median over the timed steps (HIP events between steps on the stream the kernels run on); the
    # mean over the same steps, from the host clock around the whole region, is reported next to it
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms_per_step = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])
    ms_per_step_mean = 1e3 * elapsed / args.steps
    tokens_per_s = w.B * w.N / (1e-3 * ms_per_step)
    proj, U, bytes_th = algorithmic_counts(w)
    token_heads = w.B * w.H * w.N
    step_flops = (3 * proj + 6 * U) * token_heads
    step_bytes = bytes_th * token_heads
    if args.forward_only:       # the forward pass alone: Proj + 2 U, and Q, K, V read, O and den written
        step_flops = (proj + 2 * U) * token_heads
        step_bytes = (4 * w.d * (2 if w.dtype == "bf16" else 4) + 4) * token_heads

    roofline = None
    kernels = {}
    if prof:
        shares = kernel_shares(w)
        table, table_note = measured_traffic(w) if family == 2 else (None, "no counter summary for the generic kernels")
        mfma = family == 2
        flop_peak = PEAK_BF16_FLOPS if mfma else PEAK_FP32_VECTOR_FLOPS
        for name, (ms, n) in prof.items():
            kernels[name] = {"avg_ms": ms / n, "launches_per_step": n / args.steps, "ms_per_step": ms / args.steps}
            flops, nbytes = shares.get(name, (0.0, 0.0))
            if flops or nbytes:
                kernels[name]["frac_of_%s_roof" % ("mfma" if mfma else "alu")] = flops * token_heads / (1e-3 * ms / n) / flop_peak
                kernels[name]["frac_of_hbm_roof"] = nbytes * token_heads / (1e-3 * ms / n) / PEAK_HBM_BYTES
        name = max(prof, key=lambda k: prof[k][0])
        avg_s = 1e-3 * prof[name][0] / prof[name][1]
        flops, nbytes = (x * token_heads for x in shares.get(name, (0.0, 0.0)))
        # the binding roof of the kernel's credited work is the one that takes longer at the published peaks
        t_flop, t_hbm = flops / flop_peak, nbytes / PEAK_HBM_BYTES
        traffic = table[name] * token_heads if table and name in table else None       # bytes per launch
        if t_hbm >= t_flop:
            roofline = {"kernel": name, "bound": "hbm", "achieved": nbytes / avg_s / 1e9, "peak": PEAK_HBM_BYTES / 1e9,
                        "unit": "GB/s", "frac": nbytes / avg_s / PEAK_HBM_BYTES}
        else:
            roofline = {"kernel": name, "bound": "mfma" if mfma else "alu", "achieved": flops / avg_s / 1e12,
                        "peak": flop_peak / 1e12, "unit": "TFLOP/s", "frac": flops / avg_s / flop_peak}
        roofline.update({"traffic": traffic, "traffic_source": table_note, "avg_launch_ms": 1e3 * avg_s,
                         "algorithmic_flops_per_launch": flops, "algorithmic_bytes_per_launch": nbytes,
                         "frac_of_hbm_roof": nbytes / avg_s / PEAK_HBM_BYTES,
                         "frac_of_%s_roof" % ("mfma" if mfma else "alu"): flops / avg_s / flop_peak})

    cpu_baseline = None
    if not args.no_cpu_baseline and not args.forward_only:
        from oracle import race_oracle as ro
        from oracle import stream as oracle_stream
        n0 = min(w.N, args.cpu_sample_tokens)
        rounded = w.dtype == "bf16"
        Wm = np.stack([ro.expand_projection(s, w.L, w.P, w.d, round_bf16=rounded) for s in seeds])
        b_sample = 1                                   # one batch element is enough for a rate
        host = [t[:b_sample, :, :n0].float().cpu().numpy().astype(np.float64) for t in (Q, K, V, dO)]
        tc = time.perf_counter()
        hq, hk = (ro.unit_rows(host[0]), ro.unit_rows(host[1])) if w.unit_qk else (host[0], host[1])
        Oo, deno = oracle_stream.forward(hq, hk, host[2], Wm, w.sharpening, w.L, w.P, w.causal)
        go = oracle_stream.backward(hq, hk, host[2], Wm, w.sharpening, w.L, w.P, w.causal, Oo, deno, host[3])
        if w.unit_qk:
            go = (ro.unit_rows_vjp(host[0], go[0]), ro.unit_rows_vjp(host[1], go[1]), go[2])
        cpu_s = time.perf_counter() - tc
        cpu_baseline = {"value": b_sample * n0 / cpu_s, "unit": "tokens/s", "cores": oracle_stream.threads(),
                        "kind": "oracle",
                        "sample": "first %d tokens of batch element 0 (all %d heads), fwd+bwd, fp64, %.1f s"
                                  % (n0, w.H, cpu_s)}
        if w.causal:
            # causal: the first n0 outputs depend on the first n0 tokens only, so the sample doubles as a
            # parity check of the benchmarked launch configuration (dK, dV of a prefix do not have this property)
            def err(g, r):
                g = g[:b_sample, :, :n0].float().cpu().numpy().astype(np.float64)
                return float(np.abs(g - r).max() / np.abs(r).max())
            sys.stderr.write("prefix parity vs oracle: O %.2e den %.2e dQ %.2e\n"
                             % (err(O, Oo), err(den, deno), err(dQ, go[0])))

    out = {
        "metric": ("RACE attn forward tokens/sec (not the headline metric)" if args.forward_only else
                   "RACE attn fwd+bwd tokens/sec at N=1M-12M (B=1,H=4,d=128); % MFMA/HBM roof"),
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_mean": ms_per_step_mean, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d": w.d, "L": w.L, "P": w.P,
                   "sharpening": w.sharpening, "causal": w.causal, "unit_qk": w.unit_qk, "kernel_family": family,
                   "backward": None if args.forward_only else ("race_attn_bwd" if args.bwd_recompute else "race_attn_bwd_saved")},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "step_roofline": {"algorithmic_tflop": step_flops / 1e12, "algorithmic_gb": step_bytes / 1e9,
                          "bound": "hbm" if step_bytes / PEAK_HBM_BYTES >= step_flops / (PEAK_BF16_FLOPS if family == 2 else PEAK_FP32_VECTOR_FLOPS) else ("mfma" if family == 2 else "alu"),
                          "frac_of_%s_roof" % ("mfma" if family == 2 else "alu"): step_flops / (1e-3 * ms_per_step) / (PEAK_BF16_FLOPS if family == 2 else PEAK_FP32_VECTOR_FLOPS),
                          "frac_of_hbm_roof": step_bytes / (1e-3 * ms_per_step) / PEAK_HBM_BYTES},
        "attainable": attainable,
        "kernels": kernels,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
