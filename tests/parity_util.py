"""Shared helpers of the GPU parity tests: run the HIP path through the C-ABI binding, run the oracle on
the same (rounded) inputs, and compare with the error measure of the build's tolerance statement."""
from __future__ import annotations

import numpy as np
import torch

import paper_2510_04008_amd as ra
from oracle import race_oracle as ro
from oracle import stream as oracle_stream
from paper_2510_04008_amd import synth

# max |gpu - oracle| / max |oracle| per output tensor
TOL = {"f32": 1e-4, "bf16": 2e-2}


def desc_of(w: synth.Workload):
    return ra.make_desc(w.B, w.H, w.N, w.d, w.L, w.P, w.sharpening, w.causal,
                        ra.RACE_F32 if w.dtype == "f32" else ra.RACE_BF16, w.chunk, w.unit_qk)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def oracle_w(w: synth.Workload, seeds):
    return np.stack([ro.expand_projection(s, w.L, w.P, w.d, round_bf16=(w.dtype == "bf16")) for s in seeds])


def rel_err(gpu: torch.Tensor, ref: np.ndarray, floor: float = 0.0) -> float:
    """floor: lower bound of the scale, for tensors that are zero in exact arithmetic."""
    g = to_f64(gpu)
    assert np.isfinite(g).all(), "non-finite values in GPU result"
    scale = max(np.abs(ref).max(), floor)
    return float(np.abs(g - ref).max() / (scale if scale > 0 else 1.0))


class ErrAcc:
    """Error measures of one output tensor, accumulated over slices along the token axis (axis 2):
    linf: max |gpu - oracle| / max |oracle| over the whole tensor (the build's tolerance statement);
    l2  : |gpu - oracle|_2 / |oracle|_2;
    blk : the largest of the same max-ratio taken per (batch, head, block of 1024 tokens) -- late rows of a causal
          output are much smaller than its first rows, and the tensor-wide ratio is blind to them."""

    BLOCK = 1024

    def __init__(self):
        self.max_diff = self.max_ref = self.sq_diff = self.sq_ref = self.blk = 0.0
        self.worst_block = None
        self.tokens = 0

    def update(self, gpu, ref: np.ndarray, t0: int = 0):
        g = to_f64(gpu) if isinstance(gpu, torch.Tensor) else np.asarray(gpu, dtype=np.float64)
        assert g.shape == ref.shape, (g.shape, ref.shape)
        assert np.isfinite(g).all(), "non-finite values in GPU result"
        diff = np.abs(g - ref)
        self.max_diff = max(self.max_diff, float(diff.max(initial=0.0)))
        self.max_ref = max(self.max_ref, float(np.abs(ref).max(initial=0.0)))
        self.sq_diff += float((diff * diff).sum())
        self.sq_ref += float((ref * ref).sum())
        n = ref.shape[2]
        for a in range(0, n, self.BLOCK):
            dm = diff[:, :, a:a + self.BLOCK].reshape(ref.shape[0], ref.shape[1], -1).max(axis=2)
            rm = np.abs(ref[:, :, a:a + self.BLOCK]).reshape(ref.shape[0], ref.shape[1], -1).max(axis=2)
            ratio = np.where(rm > 0, dm / np.where(rm > 0, rm, 1.0), 0.0)
            if ratio.max() > self.blk:
                self.blk = float(ratio.max())
                self.worst_block = t0 + a
        self.tokens += n
        return self

    @property
    def linf(self):
        return self.max_diff / (self.max_ref if self.max_ref > 0 else 1.0)

    @property
    def l2(self):
        return (self.sq_diff / self.sq_ref) ** 0.5 if self.sq_ref > 0 else self.sq_diff ** 0.5

    def __str__(self):
        return "linf=%.2e l2=%.2e blk=%.2e@%s" % (self.linf, self.l2, self.blk, self.worst_block)


def run_gpu(w: synth.Workload, tensors=None, seeds=None, saved=False, fwd_results=None):
    """One forward and one backward pass through the C ABI.  saved: the backward pass reads the workspace the
    forward pass left behind (race_attn_bwd_saved), the pair of calls the benchmark times.  fwd_results: callable
    (O, den) -> (O, den) that the backward pass is given instead of the forward pass's own outputs (the backward pass
    is a function of Q, K, V, O, den and dO; see check_case)."""
    Q, K, V, dO = tensors if tensors is not None else synth.make_inputs(w, "cuda")
    seeds = seeds if seeds is not None else synth.projection_seeds(w)
    d = desc_of(w)
    ws = torch.empty(max(ra.race_attn_workspace_bytes(d), 256), dtype=torch.uint8, device="cuda") if saved else None
    O, den = ra.race_attn_fwd(d, Q, K, V, seeds, workspace=ws)
    O_in, den_in = fwd_results(O, den) if fwd_results is not None else (O, den)
    if saved:
        dQ, dK, dV = ra.race_attn_bwd_saved(d, Q, K, V, O_in, den_in, dO, seeds, ws)
    else:
        dQ, dK, dV = ra.race_attn_bwd(d, Q, K, V, O_in, den_in, dO, seeds)
    torch.cuda.synchronize()
    return dict(Q=Q, K=K, V=V, dO=dO, O=O, den=den, O_in=O_in, den_in=den_in, dQ=dQ, dK=dK, dV=dV, seeds=seeds)


def oracle_forward(w: synth.Workload, Q, K, V, seeds):
    """The oracle's forward pass on the (rounded) device inputs.  Returns O, den (fp64) and what it was run on."""
    W = oracle_w(w, seeds)
    Q, K, V = (to_f64(t) for t in (Q, K, V))
    # the unit-norm option is the map x -> x / |x| in front of the layer and its chain rule behind the backward pass
    Qu, Ku = (ro.unit_rows(Q), ro.unit_rows(K)) if w.unit_qk else (Q, K)
    O, den = oracle_stream.forward(Qu, Ku, V, W, w.sharpening, w.L, w.P, w.causal)
    return O, den, dict(W=W, Q=Q, K=K, V=V, Qu=Qu, Ku=Ku)


def oracle_backward(w: synth.Workload, ctx, O, den, dO, with_beta=False):
    """The oracle's backward pass given the forward results O, den (any arrays of the right shape: the backward pass
    is a function of Q, K, V, O, den, dO)."""
    out = oracle_stream.backward(ctx["Qu"], ctx["Ku"], ctx["V"], ctx["W"], w.sharpening, w.L, w.P, w.causal,
                                 O, den, to_f64(dO), with_beta=with_beta)
    dQ, dK, dV = out[:3]
    if w.unit_qk:
        dQ, dK = ro.unit_rows_vjp(ctx["Q"], dQ), ro.unit_rows_vjp(ctx["K"], dK)
    return (dQ, dK, dV, out[3]) if with_beta else (dQ, dK, dV)


def rounded_forward_results(w: synth.Workload, O: np.ndarray, den: np.ndarray):
    """The oracle's O and Den as tensors of the layer's storage types (O in the element type, den in fp32): what a
    caller of the backward pass holds after an exact forward pass."""
    return (torch.from_numpy(O).to(torch.float32).to(w.torch_dtype).cuda().contiguous(),
            torch.from_numpy(den).to(torch.float32).cuda().contiguous())


# Bound on the max-ratio per block of 1024 tokens (ErrAcc.blk), as a multiple of the tensor-wide tolerance: every block
# is held to the tolerance itself.
BLOCK_FACTOR = 1.0


def check_case(w: synth.Workload, tensors=None, tol=None, verbose=True, floors=None, saved=False):
    """Forward: the kernels' O and Den against the oracle's.  Backward: the kernels and the oracle are both given the
    oracle's O and Den rounded to the storage types (bf16/fp32 O, fp32 Den), so that dQ, dK, dV are compared as what
    they are, a function of (Q, K, V, O, Den, dO), on identical arguments; gradients of the first rows of a causal
    sequence are ill-conditioned in O (terms scaled by 1/Den cancel when O_i equals the one value it averages), and
    feeding the two sides different roundings of O would measure that conditioning, not the kernels."""
    tol = tol or TOL[w.dtype]
    floors = floors or {}
    tensors = tensors if tensors is not None else synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    O_r, den_r, ctx = oracle_forward(w, tensors[0], tensors[1], tensors[2], seeds)
    assert den_r.min() > 1e-30
    O_in, den_in = rounded_forward_results(w, O_r, den_r)
    g = run_gpu(w, tensors, seeds, saved=saved, fwd_results=lambda O, den: (O_in, den_in))
    dQ, dK, dV = oracle_backward(w, ctx, to_f64(O_in), to_f64(den_in), g["dO"])
    r = dict(O=O_r, den=den_r, dQ=dQ, dK=dK, dV=dV)
    accs = {}
    for n in ("O", "den", "dQ", "dK", "dV"):
        gt, rt = (g[n].unsqueeze(-1), r[n][..., None]) if n == "den" else (g[n], r[n])
        accs[n] = ErrAcc().update(gt, rt)
        if floors.get(n, 0.0) > accs[n].max_ref:          # tensors that are zero in exact arithmetic: see the caller
            accs[n].max_ref = floors[n]
            accs[n].sq_ref = max(accs[n].sq_ref, floors[n] ** 2 * rt.size)
            accs[n].blk = 0.0
    errs = {n: a.linf for n, a in accs.items()}
    if verbose:
        print("%s: family=%d " % (w.name, ra.race_attn_kernel_family(desc_of(w))) +
              "  ".join("%s[%s]" % kv for kv in accs.items()), flush=True)
    for n, a in accs.items():
        assert a.linf < tol, "%s: %s max-ratio %.3e >= %.1e" % (w.name, n, a.linf, tol)
        assert a.l2 < tol, "%s: %s relative l2 error %.3e >= %.1e" % (w.name, n, a.l2, tol)
        assert a.blk < BLOCK_FACTOR * tol, "%s: %s max-ratio %.3e in the block at token %s" % (w.name, n, a.blk, a.worst_block)
    return g, r, errs


# unit roundoff of the arithmetic the terms of a sum go through (bf16 operands of the matrix products; fp32)
UNIT_ROUNDOFF = {"bf16": 2.0 ** -9, "f32": 2.0 ** -24}
WELL_CONDITIONED = 100.0


def check_dbeta(w: synth.Workload, tol=None, verbose=True):
    """Cotangent of the temperature per (batch, head) from race_attn_bwd_beta against the oracle, both given the
    oracle's O and Den rounded to the storage types; also checks that asking for it leaves dQ, dK, dV bit-identical.
    dbeta is one sum of ~N L P terms of both signs per (batch, head).  Its condition number is
    cond = (sum of |terms|) / |sum| (the oracle's beta_cotangent_l1 over |dbeta|), and a path whose terms each carry
    one unit roundoff u of relative error is off by at most u * cond relative to dbeta.  Asserted:
      (1) |gpu - oracle| <= 4 u * sum |terms| for every (batch, head) -- the conditioning bound, with a factor for
          the handful of roundings a term goes through (u = 2^-9 for bf16 operands, 2^-24 for fp32);
      (2) where cond <= 100, the tensors' own measure: max |gpu - oracle| / max |oracle| below the tolerance."""
    tol = tol or TOL[w.dtype]
    tensors = synth.make_inputs(w, "cuda")
    seeds = synth.projection_seeds(w)
    O_r, den_r, ctx = oracle_forward(w, tensors[0], tensors[1], tensors[2], seeds)
    O_in, den_in = rounded_forward_results(w, O_r, den_r)
    g = run_gpu(w, tensors, seeds, fwd_results=lambda O, den: (O_in, den_in))
    d = desc_of(w)
    dQ, dK, dV, dbeta = ra.race_attn_bwd_beta(d, g["Q"], g["K"], g["V"], O_in, den_in, g["dO"], g["seeds"])
    torch.cuda.synchronize()
    for a, b in ((dQ, g["dQ"]), (dK, g["dK"]), (dV, g["dV"])):
        assert torch.equal(a, b)
    *_, ref = oracle_backward(w, ctx, to_f64(O_in), to_f64(den_in), g["dO"], with_beta=True)
    got = to_f64(dbeta)
    assert np.isfinite(got).all()
    dO = to_f64(g["dO"])
    l1 = np.array([[ro.beta_cotangent_l1(ctx["Qu"][b, h], ctx["Ku"][b, h], ctx["V"][b, h], ctx["W"][h], w.sharpening, w.L, w.P,
                                         w.causal, dO[b, h]) for h in range(w.H)] for b in range(w.B)])
    assert (l1 >= np.abs(ref) * (1 - 1e-9)).all()
    cond = float((l1 / np.abs(ref)).max())
    err_terms = float((np.abs(got - ref) / l1).max())
    err_max = float(np.abs(got - ref).max() / np.abs(ref).max())
    if verbose:
        print("%s: dbeta error %.2e of max |dbeta| = %.3e; %.2e of the terms' l1 norm; condition number %.0f"
              % (w.name, err_max, np.abs(ref).max(), err_terms, cond), flush=True)
    assert err_terms <= 4 * UNIT_ROUNDOFF[w.dtype], (w.name, err_terms)
    if cond <= WELL_CONDITIONED:
        assert err_max < tol, "%s: dbeta err %.3e >= %.1e at condition number %.0f" % (w.name, err_max, tol, cond)
    return dbeta, ref
