"""fp64 CPU oracle for RACE Attention (forward and backward).

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct statement of
what the layer computes, written from the paper.  It shares no code with the HIP
library and must never be imported by the product path; only the tests, the smoke
check and the benchmark's cpu_baseline leg may call it.

Every function works on ONE (batch, head) slice: Q, K, V are (N, d) float64 arrays
and W is the (L*P, d) projection matrix whose rows l*P .. l*P+P-1 are the P
hyperplanes of table l (Algorithm 1, step 2).

Pinned by tests/test_oracle_*.py against closed forms, brute force and finite
differences; nothing here is "parity unpinned".

Readings of the paper taken here (each is listed with its reason in the design notes):
  * beta is the single temperature of Algorithm 1/2 ("sharpening" of the interface).
  * No normalisation of Q, K and no 1/sqrt(d) scaling inside the layer (Algorithm 1, step 4); the
    unit-norm setting of the analysis (Appendix, setup of the proof of Theorem 1) is an option of the
    interface, stated here as unit_rows() in front of the layer and unit_rows_vjp() behind its backward pass.
  * Corner r of the hypercube has v_{r,t} = +1 iff bit t of r is set; t = 0 is the
    least significant bit and belongs to row l*P+0 of W.
  * The causal variant is inclusive (j <= i): Algorithm 2 adds key/value t to the
    running bucket statistics before query t reads them.
  * Den keeps the 1/L of Algorithm 1, step 7 (it cancels in O).
  * beta is trained in the paper's experiments (Section 4), so the backward functions can also
    return its cotangent; with W fixed and random it is the layer's only parameter gradient.
"""
from __future__ import annotations

import math

import numpy as np

# ----------------------------------------------------------------------------------
# Projection matrix generator (Algorithm 1, step 2: rows of W^(l) i.i.d. N(0, I_d))
# ----------------------------------------------------------------------------------
# The interface passes one 64-bit seed per head.  Both this oracle and the library
# expand a seed with the same published counter-based generator (Philox-4x32-10,
# Salmon et al., SC'11) followed by a Box-Muller transform in fp64, so that W is
# bit-identical on both sides without either side handing values to the other.

_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """Philox-4x32 with 10 rounds.  counter: 4 uint32, key: 2 uint32 -> 4 uint32."""
    c0, c1, c2, c3 = (int(x) & _MASK32 for x in counter)
    k0, k1 = (int(x) & _MASK32 for x in key)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _PHILOX_W0) & _MASK32
            k1 = (k1 + _PHILOX_W1) & _MASK32
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & _MASK32
        hi1, lo1 = p1 >> 32, p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def _box_muller(x0: int, x1: int):
    """Two u32 -> two independent N(0,1) in fp64.  u = (x + 0.5) / 2^32 lies in (0, 1)."""
    u1 = (x0 + 0.5) * (1.0 / 4294967296.0)
    u2 = (x1 + 0.5) * (1.0 / 4294967296.0)
    rad = math.sqrt(-2.0 * math.log(u1))
    ang = 2.0 * math.pi * u2
    return rad * math.cos(ang), rad * math.sin(ang)


def expand_projection(seed: int, L: int, P: int, d: int, round_bf16: bool = False) -> np.ndarray:
    """W (L*P, d) for one head from its 64-bit seed, as float32 values held in float64.

    Element e = row*d + col is Gaussian number (e mod 4) of Philox block e // 4
    (counter = (block_lo, block_hi, 0, 0), key = (seed_lo, seed_hi)); a block's four
    words give two Box-Muller pairs.  Values are rounded fp64 -> fp32 (nearest even);
    with round_bf16 they are rounded once more, fp32 -> bf16 (nearest even), which is
    what a bf16 tensor path multiplies with.
    """
    n = L * P * d
    key = (seed & _MASK32, (seed >> 32) & _MASK32)
    out = np.empty(n, dtype=np.float64)
    for blk in range((n + 3) // 4):
        x = philox4x32_10((blk & _MASK32, (blk >> 32) & _MASK32, 0, 0), key)
        g = _box_muller(x[0], x[1]) + _box_muller(x[2], x[3])
        lo = 4 * blk
        out[lo:lo + 4] = g[: min(4, n - lo)]
    w32 = out.astype(np.float32)
    if round_bf16:
        w32 = round_to_bf16(w32)
    return w32.astype(np.float64).reshape(L * P, d)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result kept as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    bias = ((bits >> 16) & 1) + 0x7FFF
    bits = ((bits + bias) >> 16) << 16
    return (bits & 0xFFFFFFFF).astype(np.uint32).view(np.float32).reshape(x.shape)


# ----------------------------------------------------------------------------------
# Soft-LSH bucket assignment (Algorithm 1, steps 2-4)
# ----------------------------------------------------------------------------------

def corners(P: int) -> np.ndarray:
    """(R, P) matrix of hypercube corners: v[r, t] = +1 if bit t of r is set, else -1."""
    r = np.arange(1 << P)[:, None]
    t = np.arange(P)[None, :]
    return np.where((r >> t) & 1, 1.0, -1.0)


def project(X: np.ndarray, W: np.ndarray, L: int, P: int) -> np.ndarray:
    """z[i, l, t] = <W[l*P+t, :], X[i, :]>  (Algorithm 1, step 4: the argument of tanh)."""
    return (X @ W.T).reshape(X.shape[0], L, P)


def hard_codes(X: np.ndarray, W: np.ndarray, L: int, P: int) -> np.ndarray:
    """Integer bucket of the hard hash sign(W x): bit t of the code is [z_t >= 0]  (Section 3.3)."""
    z = project(X, W, L, P)
    return ((z >= 0).astype(np.int64) << np.arange(P)).sum(axis=2)


def soft_hash(X: np.ndarray, W: np.ndarray, beta: float, L: int, P: int) -> np.ndarray:
    """phi[i, l, r] = softmax_r( beta * tanh(W^(l) x_i) . v_r )   (Algorithm 1, step 4)."""
    u = np.tanh(project(X, W, L, P))                      # (N, L, P)
    logits = beta * np.einsum("nlt,rt->nlr", u, corners(P))
    logits -= logits.max(axis=2, keepdims=True)
    e = np.exp(logits)
    return e / e.sum(axis=2, keepdims=True)


# ----------------------------------------------------------------------------------
# Forward
# ----------------------------------------------------------------------------------

def kernel_matrix(Q, K, W, beta, L, P) -> np.ndarray:
    """S_hat[i, j] = (1/L) sum_l phi_l(Q_i) . phi_l(K_j)   (Section 3.3 / Appendix, RACE kernel)."""
    pq = soft_hash(Q, W, beta, L, P)
    pk = soft_hash(K, W, beta, L, P)
    return np.einsum("ilr,jlr->ij", pq, pk) / L


def forward_quadratic(Q, K, V, W, beta, L, P, causal):
    """The definition: O = D^-1 (M o S_hat) V with the explicit N x N kernel matrix.

    Returns (O, Den) where Den_i = sum_j M_ij S_hat_ij.  M is all-ones, or the inclusive
    lower triangle in the causal case.
    """
    S = kernel_matrix(Q, K, W, beta, L, P)
    if causal:
        S = np.tril(S)
    den = S.sum(axis=1)
    return (S @ V) / den[:, None], den


def forward_linear(Q, K, V, W, beta, L, P):
    """Algorithm 1 (non-causal), steps 5, 7 and 8, as written."""
    pq = soft_hash(Q, W, beta, L, P)
    pk = soft_hash(K, W, beta, L, P)
    N, d = V.shape
    num = np.zeros((N, d))
    den = np.zeros(N)
    for l in range(L):
        A = pk[:, l, :].T @ np.ones(N)          # (R,)
        B = pk[:, l, :].T @ V                   # (R, d)
        num += pq[:, l, :] @ B
        den += pq[:, l, :] @ A
    num /= L
    den /= L
    return num / den[:, None], den


def forward_streaming(Q, K, V, W, beta, L, P):
    """Algorithm 2 (causal), one left-to-right scan per table: update with token t, then read."""
    pq = soft_hash(Q, W, beta, L, P)
    pk = soft_hash(K, W, beta, L, P)
    N, d = V.shape
    R = 1 << P
    num = np.zeros((N, d))
    den = np.zeros(N)
    for l in range(L):
        A = np.zeros(R)
        B = np.zeros((R, d))
        for t in range(N):
            A += pk[t, l, :]
            B += np.outer(pk[t, l, :], V[t])
            num[t] += pq[t, l, :] @ B
            den[t] += pq[t, l, :] @ A
    num /= L
    den /= L
    return num / den[:, None], den


def forward_hard(Q, K, V, W, L, P, causal):
    """Hard RACE (Section 3.3: the hash h(x) = sign(W x) before it is softened; the limit beta -> infinity of
    Algorithms 1/2).  Every table keeps per-bucket counters A (keys seen) and B (their summed values); key j
    goes to bucket hard_codes(K_j) of every table, query i reads the counters of its own buckets:
    Num_i = (1/L) sum_l B_l[code_l(Q_i)], Den_i = (1/L) sum_l A_l[code_l(Q_i)], O_i = Num_i / Den_i.
    Causal: key i is added before query i reads (Algorithm 2).  A query whose buckets are all empty has
    Den_i = 0; O_i is defined as 0 then (the paper does not say; the soft assignment never gets there)."""
    cq, ck = hard_codes(Q, W, L, P), hard_codes(K, W, L, P)
    N, d = V.shape
    R = 1 << P
    A = np.zeros((L, R))
    B = np.zeros((L, R, d))
    num = np.zeros((N, d))
    den = np.zeros(N)
    tables = np.arange(L)
    if not causal:
        for j in range(N):
            A[tables, ck[j]] += 1.0
            B[tables, ck[j]] += V[j]
    for i in range(N):
        if causal:
            A[tables, ck[i]] += 1.0
            B[tables, ck[i]] += V[i]
        num[i] = B[tables, cq[i]].sum(axis=0) / L
        den[i] = A[tables, cq[i]].sum() / L
    O = np.where(den[:, None] > 0, num / np.where(den > 0, den, 1.0)[:, None], 0.0)
    return O, den


def bucket_statistics(K, V, W, beta, L, P):
    """Final (all-N) per-table statistics A (L, R) and B (L, R, d) of Algorithm 1, step 5."""
    pk = soft_hash(K, W, beta, L, P)
    A = pk.sum(axis=0)
    B = np.einsum("nlr,nc->lrc", pk, V)
    return A, B


def decode_step(state, q, k, v, W, beta, L, P):
    """One iteration of Algorithm 2's loop with the bucket statistics as the carried state (the layer's
    counterpart of a key/value cache: its size does not grow with the context).  state: (L, R, d+1)
    float64, [B | A] per bucket row, updated in place with (k, v); returns the output row of q and Den."""
    d = q.shape[0]
    pk = soft_hash(k[None, :], W, beta, L, P)[0]          # (L, R)
    pq = soft_hash(q[None, :], W, beta, L, P)[0]
    state[:, :, :d] += pk[:, :, None] * v[None, None, :]
    state[:, :, d] += pk
    num = np.einsum("lr,lrc->c", pq, state[:, :, :d]) / L
    den = float((pq * state[:, :, d]).sum()) / L
    return num / den, den


# ----------------------------------------------------------------------------------
# Backward (the paper trains through the soft assignment by automatic differentiation
# and prints no gradient; both forms below are derived from Algorithms 1/2 and are
# checked against central finite differences)
# ----------------------------------------------------------------------------------

def _soft_hash_vjp(X, W, beta, L, P, dphi):
    """Pull a cotangent dphi (N, L, R) back through softmax, the corner logits, tanh and W."""
    u = np.tanh(project(X, W, L, P))
    phi = soft_hash(X, W, beta, L, P)
    ds = phi * (dphi - (phi * dphi).sum(axis=2, keepdims=True))      # softmax
    du = beta * np.einsum("nlr,rt->nlt", ds, corners(P))             # logits = beta u.v_r
    dz = du * (1.0 - u * u)                                          # tanh
    return dz.reshape(X.shape[0], L * P) @ W                         # z = W x


def _soft_hash_vjp_beta(X, W, beta, L, P, dphi) -> float:
    """Cotangent of the temperature beta (trained in the paper's experiments, Section 4): the corner
    logits are beta * (u . v_r), so d(beta) = sum over tokens, tables and corners of ds_r (u . v_r)."""
    u = np.tanh(project(X, W, L, P))
    phi = soft_hash(X, W, beta, L, P)
    ds = phi * (dphi - (phi * dphi).sum(axis=2, keepdims=True))
    return float(np.einsum("nlr,rt,nlt->", ds, corners(P), u))


def backward_quadratic(Q, K, V, W, beta, L, P, causal, dO, with_beta: bool = False):
    """Gradients of sum(dO * O) through the explicit N x N form.  Returns dQ, dK, dV
    (and d(beta) if with_beta)."""
    pq = soft_hash(Q, W, beta, L, P)
    pk = soft_hash(K, W, beta, L, P)
    S = np.einsum("ilr,jlr->ij", pq, pk) / L
    M = np.tril(np.ones_like(S)) if causal else np.ones_like(S)
    S = S * M
    den = S.sum(axis=1)
    Amat = S / den[:, None]                         # attention weights, rows sum to 1
    O = Amat @ V
    dV = Amat.T @ dO
    # O_i = sum_j S_ij V_j / den_i  =>  dS_ij = M_ij (V_j - O_i).dO_i / den_i
    dS = M * ((dO @ V.T) - (dO * O).sum(axis=1)[:, None]) / den[:, None]
    dpq = np.einsum("ij,jlr->ilr", dS, pk) / L
    dpk = np.einsum("ij,ilr->jlr", dS, pq) / L
    dQ = _soft_hash_vjp(Q, W, beta, L, P, dpq)
    dK = _soft_hash_vjp(K, W, beta, L, P, dpk)
    if with_beta:
        return dQ, dK, dV, _soft_hash_vjp_beta(Q, W, beta, L, P, dpq) + _soft_hash_vjp_beta(K, W, beta, L, P, dpk)
    return dQ, dK, dV


def backward_streaming(Q, K, V, W, beta, L, P, causal, dO, with_beta: bool = False):
    """Gradients in linear time with bucket-sized state only (nothing N x N, nothing N x R kept
    beyond phi itself).  Pass 1 runs left to right with the prefix statistics (A, B) and gives
    the cotangent of phi_Q; pass 2 runs right to left with the suffix statistics (dA, dB) of
    the read-out cotangents and gives dV and the cotangent of phi_K.  Non-causal: both
    statistics are the all-N totals.
    """
    pq = soft_hash(Q, W, beta, L, P)
    pk = soft_hash(K, W, beta, L, P)
    N, d = V.shape
    R = 1 << P
    O, den = (forward_streaming if causal else forward_linear)(Q, K, V, W, beta, L, P)
    e = den * L                                           # un-averaged normaliser
    gn = dO / e[:, None]                                  # cotangent of the un-averaged numerator
    ge = -(dO * O).sum(axis=1) / e                        # cotangent of the un-averaged normaliser
    dpq = np.zeros_like(pq)
    dpk = np.zeros_like(pk)
    dV = np.zeros_like(V)
    for l in range(L):
        if causal:
            A = np.zeros(R)
            B = np.zeros((R, d))
            for i in range(N):
                A += pk[i, l]
                B += np.outer(pk[i, l], V[i])
                dpq[i, l] = B @ gn[i] + A * ge[i]
            dA = np.zeros(R)
            dB = np.zeros((R, d))
            for j in range(N - 1, -1, -1):
                dA += pq[j, l] * ge[j]
                dB += np.outer(pq[j, l], gn[j])
                dV[j] += pk[j, l] @ dB
                dpk[j, l] = dB @ V[j] + dA
        else:
            A = pk[:, l].sum(axis=0)
            B = pk[:, l].T @ V
            dA = pq[:, l].T @ ge
            dB = pq[:, l].T @ gn
            dpq[:, l] = gn @ B.T + np.outer(ge, A)
            dV += pk[:, l] @ dB
            dpk[:, l] = V @ dB.T + dA[None, :]
    dQ = _soft_hash_vjp(Q, W, beta, L, P, dpq)
    dK = _soft_hash_vjp(K, W, beta, L, P, dpk)
    if with_beta:
        return dQ, dK, dV, _soft_hash_vjp_beta(Q, W, beta, L, P, dpq) + _soft_hash_vjp_beta(K, W, beta, L, P, dpk)
    return dQ, dK, dV


def beta_cotangent_terms(Q, K, V, W, beta, L, P, causal, dO):
    """The terms ds_r (u . v_r), one per (token of Q or K, table, hyperplane), whose sum is d(loss)/d(beta) (N x N
    form; Algorithm 1, step 4: the logit of corner r is beta * (tanh(W x) . v_r)).  Returns (terms of Q, terms of K),
    each (N, L, P)."""
    pq = soft_hash(Q, W, beta, L, P)
    pk = soft_hash(K, W, beta, L, P)
    S = np.einsum("ilr,jlr->ij", pq, pk) / L
    M = np.tril(np.ones_like(S)) if causal else np.ones_like(S)
    S = S * M
    den = S.sum(axis=1)
    O = (S / den[:, None]) @ V
    dS = M * ((dO @ V.T) - (dO * O).sum(axis=1)[:, None]) / den[:, None]
    out = []
    for X, phi, dphi in ((Q, pq, np.einsum("ij,jlr->ilr", dS, pk) / L), (K, pk, np.einsum("ij,ilr->jlr", dS, pq) / L)):
        u = np.tanh(project(X, W, L, P))
        ds = phi * (dphi - (phi * dphi).sum(axis=2, keepdims=True))
        out.append(np.einsum("nlr,rt->nlt", ds, corners(P)) * u)
    return out[0], out[1]


def beta_cotangent_l1(Q, K, V, W, beta, L, P, causal, dO) -> float:
    """Sum of the absolute values of those terms: the scale against which rounding errors of an implementation add up
    when the terms cancel."""
    tq, tk = beta_cotangent_terms(Q, K, V, W, beta, L, P, causal, dO)
    return float(np.abs(tq).sum() + np.abs(tk).sum())


def finite_difference_beta(Q, K, V, W, beta, L, P, causal, dO, h: float = 1e-6) -> float:
    """Central difference of loss = sum(dO * O) with respect to the temperature beta."""
    def loss(b):
        o, _ = forward_quadratic(Q, K, V, W, b, L, P, causal)
        return float((dO * o).sum())
    return (loss(beta + h) - loss(beta - h)) / (2 * h)


def finite_difference(Q, K, V, W, beta, L, P, causal, dO, which: str, index, h: float = 1e-6) -> float:
    """Central difference of loss = sum(dO * O) with respect to one entry of Q, K or V."""
    def loss(q, k, v):
        o, _ = forward_quadratic(q, k, v, W, beta, L, P, causal)
        return float((dO * o).sum())
    T = {"Q": Q, "K": K, "V": V}
    plus = {n: a.copy() for n, a in T.items()}
    minus = {n: a.copy() for n, a in T.items()}
    plus[which][index] += h
    minus[which][index] -= h
    return (loss(plus["Q"], plus["K"], plus["V"]) - loss(minus["Q"], minus["K"], minus["V"])) / (2 * h)


# ----------------------------------------------------------------------------------
# Optional unit-norm queries and keys (Appendix, setup of the proof of Theorem 1: |Q_i| = |K_j| = 1)
# ----------------------------------------------------------------------------------
# The interface can divide every row of Q and K by its Euclidean norm before Algorithm 1/2 sees it.
# Rows shorter than UNIT_EPS are divided by UNIT_EPS instead (a zero row stays zero).

UNIT_EPS = 1e-12


def unit_rows(X: np.ndarray) -> np.ndarray:
    """x / max(|x|, UNIT_EPS) for every row of X (..., d)."""
    n = np.maximum(np.sqrt((X * X).sum(axis=-1, keepdims=True)), UNIT_EPS)
    return X / n


def unit_rows_vjp(X: np.ndarray, dXhat: np.ndarray) -> np.ndarray:
    """Cotangent of X given the cotangent of unit_rows(X): the Jacobian of x -> x / |x| is
    (I - xhat xhat^T) / |x|, the projection onto the tangent space of the sphere, scaled; a row
    below UNIT_EPS was only divided by a constant."""
    norm = np.sqrt((X * X).sum(axis=-1, keepdims=True))
    n = np.maximum(norm, UNIT_EPS)
    xhat = X / n
    radial = (xhat * dXhat).sum(axis=-1, keepdims=True)
    return np.where(norm >= UNIT_EPS, (dXhat - xhat * radial) / n, dXhat / n)


# ----------------------------------------------------------------------------------
# Multi-head convenience wrappers (loop over batch and head; W is shared by the batch)
# ----------------------------------------------------------------------------------

def forward(Q, K, V, Ws, beta, L, P, causal):
    """Q, K, V: (B, H, N, d) float64; Ws: list of H matrices (L*P, d).  Returns O, Den."""
    Bn, H, N, d = Q.shape
    O = np.empty_like(Q)
    den = np.empty((Bn, H, N))
    for b in range(Bn):
        for h in range(H):
            if causal:
                O[b, h], den[b, h] = forward_streaming(Q[b, h], K[b, h], V[b, h], Ws[h], beta, L, P)
            else:
                O[b, h], den[b, h] = forward_linear(Q[b, h], K[b, h], V[b, h], Ws[h], beta, L, P)
    return O, den


def backward(Q, K, V, Ws, beta, L, P, causal, dO, with_beta: bool = False):
    """Returns dQ, dK, dV (and, if with_beta, d(beta) per (batch, head): shape (B, H); the derivative
    with respect to one beta shared by everything is their sum)."""
    Bn, H, N, d = Q.shape
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    dbeta = np.zeros((Bn, H))
    for b in range(Bn):
        for h in range(H):
            dQ[b, h], dK[b, h], dV[b, h], dbeta[b, h] = backward_streaming(
                Q[b, h], K[b, h], V[b, h], Ws[h], beta, L, P, causal, dO[b, h], with_beta=True)
    return (dQ, dK, dV, dbeta) if with_beta else (dQ, dK, dV)
