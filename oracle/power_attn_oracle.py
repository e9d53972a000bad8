"""Float64 CPU oracle for causal power attention (test infrastructure, NOT the product).

This file is the checker the HIP library is compared against.  It is slow on purpose:
plain numpy in float64, one head at a time, no blocking or fusion beyond what the
definitions state.  Only tests, the smoke check and the benchmark's ``cpu_baseline``
leg may import it; the product path never does, and it shares no code with the HIP
kernels.

What it follows (arXiv 2507.04239):
  * power attention, Sec. 4 Eq. (7):  Y_i = sum_{j<=i} (Q_i . K_j)^p V_j
  * normalisation by the sum of the attention scores, Sec. 2 "Normalization" and the
    fused query-state formula of App. E.4:  O_i = Y_i / sum_{j<=i} (Q_i . K_j)^p
  * causal mask includes the diagonal (the sums of Sec. 2 Eq. (3) and Sec. 4 Eq. (7)
    run j = 1..i)
  * TPOW (Lemma 4.1), SPOW (Lemma 4.2), TSPOW (Sec. 4.1.1)
  * linear-attention recurrent form (Sec. 2 Eq. (6)) and chunked form (Sec. 2
    "Chunked form", App. A), update-state / query-state (Sec. 4.1 Eq. (10), App. E.2/E.4)
  * the backward pass is not in the paper; it is derived here from the definition
    of the forward pass and pinned by finite differences in the tests.
  * gating (Sec. 2 "Gating", App. E.2 / E.3): per-timestep log-gates, see the section below.
  * the single-token decode step: one iteration of the recurrent form with the state kept
    between calls.

Conventions: arrays of one head are 2-D, ``Q, K: [T, d]``, ``V, G: [T, v]``.  ``scale``
multiplies the score before the power, ``s_ij = scale * (q_i . k_j)``.  A row whose
denominator is exactly zero gets output zero and contributes no gradient (the paper
is silent; this is this library's convention).

Every function here is pinned by tests that do not call it to produce their own
expected values (closed forms, hand-computed fixtures, the paper's printed numbers,
pure-Python brute force, finite differences); nothing here is "parity unpinned".
"""
from __future__ import annotations

import functools
import itertools
import math

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# Embeddings (Sec. 4, Lemma 4.1 / 4.2; Sec. 4.1.1)
# --------------------------------------------------------------------------------------

def ndmi(n: int, p: int) -> np.ndarray:
    """Non-decreasing multi-indices (i_1 <= ... <= i_p) over {0..n-1}, lexicographic.

    Lemma 4.2 defines the set; the order is not fixed by the paper, lexicographic is
    this oracle's choice (it matches the order of the worked SPOW examples).
    Returns an int array [C(n+p-1, p), p].
    """
    if p == 0:
        return np.zeros((1, 0), dtype=np.int64)
    rows = list(itertools.combinations_with_replacement(range(n), p))
    return np.asarray(rows, dtype=np.int64).reshape(len(rows), p)


def multiplicity(index_row) -> int:
    """p! / prod_k hist_k(i)!  -- the number of distinct orderings of a multi-index
    (the quantity under the square root in Lemma 4.2)."""
    p = len(index_row)
    m = math.factorial(p)
    for cnt in np.unique(np.asarray(index_row), return_counts=True)[1]:
        m //= math.factorial(int(cnt))
    return m


@functools.lru_cache(maxsize=16)
def _ndmi_and_weights(d: int, p: int):
    """(ndmi(d, p), sqrt of each row's multiplicity), memoised: building the table for
    p=4, d=32 (52360 rows) takes about a second."""
    idx = ndmi(d, p)
    w = np.sqrt(np.asarray([multiplicity(r) for r in idx], dtype=F64))
    return idx, w


def dim_tpow(d: int, p: int) -> int:
    """Lemma 4.1: TPOW_p maps R^d to R^(d^p)."""
    return d ** p


def dim_spow(d: int, p: int) -> int:
    """Lemma 4.2 statement 1: D = C(d + p - 1, p)."""
    return math.comb(d + p - 1, p)


def dim_tspow(d: int, p: int, d_tile: int) -> int:
    """Sec. 4.1.1: D = C(d/d_tile + p - 1, p) * d_tile^p."""
    assert d % d_tile == 0
    return math.comb(d // d_tile + p - 1, p) * d_tile ** p


def tpow(x: np.ndarray, p: int) -> np.ndarray:
    """Lemma 4.1: the flattened p-fold tensor power of x (row-major multi-index order).
    ``x`` may be [d] or [T, d]; the embedding acts on the last axis."""
    x = np.asarray(x, dtype=F64)
    out = np.ones(x.shape[:-1] + (1,), dtype=F64)
    for _ in range(p):
        out = (out[..., :, None] * x[..., None, :]).reshape(x.shape[:-1] + (-1,))
    return out


def spow(x: np.ndarray, p: int) -> np.ndarray:
    """Lemma 4.2: entries sqrt(p!/prod_k hist_k(i)!) * prod_k x_{i_k} over the
    non-decreasing multi-indices i, in lexicographic order."""
    x = np.asarray(x, dtype=F64)
    d = x.shape[-1]
    idx, w = _ndmi_and_weights(d, p)
    out = np.ones(x.shape[:-1] + (idx.shape[0],), dtype=F64)
    for z in range(p):
        out = out * x[..., idx[:, z]]
    return out * w


def tspow(x: np.ndarray, p: int, d_tile: int) -> np.ndarray:
    """Sec. 4.1.1 tiled symmetric power: x is cut into d/d_tile sub-vectors; for every
    non-decreasing *tile* multi-index (t_1 <= ... <= t_p) the block
    flat(x^{t_1} (x) ... (x) x^{t_p}) of d_tile^p entries is emitted.

    The paper's text and Alg. 1/2 show no weight on the blocks; without one the inner
    product of two embeddings is not (q.k)^p.  Reading taken here: each block carries
    sqrt(multiplicity of the tile multi-index), the tile-level analogue of Lemma 4.2.
    """
    x = np.asarray(x, dtype=F64)
    d = x.shape[-1]
    assert d % d_tile == 0
    nt = d // d_tile
    blocks = []
    for lam in ndmi(nt, p):
        blk = np.ones(x.shape[:-1] + (1,), dtype=F64)
        for t in lam:
            sub = x[..., t * d_tile:(t + 1) * d_tile]
            blk = (blk[..., :, None] * sub[..., None, :]).reshape(x.shape[:-1] + (-1,))
        blocks.append(math.sqrt(multiplicity(lam)) * blk)
    return np.concatenate(blocks, axis=-1)


def spow_jacobian_transpose_apply(x: np.ndarray, g: np.ndarray, p: int) -> np.ndarray:
    """J_phi(x)^T g for phi = SPOW_p, rows of x: [T, d], g: [T, D] -> [T, d].

    d phi_r / d x_a = w_r * sum over the positions z with i_z = a of prod_{z' != z} x_{i_z'}
    (product rule applied to Lemma 4.2's entry)."""
    x = np.asarray(x, dtype=F64)
    g = np.asarray(g, dtype=F64)
    T, d = x.shape
    idx, w = _ndmi_and_weights(d, p)
    out = np.zeros((T, d), dtype=F64)
    for z in range(p):
        rest = np.ones((T, idx.shape[0]), dtype=F64)
        for z2 in range(p):
            if z2 != z:
                rest = rest * x[:, idx[:, z2]]
        contrib = g * rest * w                         # [T, D]
        onehot = np.zeros((idx.shape[0], d), dtype=F64)
        onehot[np.arange(idx.shape[0]), idx[:, z]] = 1.0
        out += contrib @ onehot                        # scatter-add over the index a = i_z
    return out


# --------------------------------------------------------------------------------------
# Attention form: the plain definition (Sec. 4 Eq. (7) + normalisation)
# --------------------------------------------------------------------------------------

def _ipow(s: np.ndarray, p: int) -> np.ndarray:
    """s^p by repeated multiplication (integer p >= 0)."""
    out = np.ones_like(s)
    for _ in range(p):
        out = out * s
    return out


def _safe_div(num: np.ndarray, den: np.ndarray) -> np.ndarray:
    """num/den with den == 0 -> 0 (zero-denominator convention of this library)."""
    den = np.asarray(den, dtype=F64)
    ok = den != 0.0
    return np.where(ok, num / np.where(ok, den, 1.0), 0.0)


def fwd_row(Q, K, V, i: int, p: int, normalize: bool = True, scale: float = 1.0):
    """One output row by the definition: returns (O_i [v], Z_i)."""
    q = np.asarray(Q[i], dtype=F64)
    Kc = np.asarray(K[: i + 1], dtype=F64)
    Vc = np.asarray(V[: i + 1], dtype=F64)
    a = _ipow(scale * (Kc @ q), p)
    N = a @ Vc
    Z = a.sum()
    if normalize:
        return (N / Z if Z != 0.0 else np.zeros_like(N)), Z
    return N, Z


def fwd_quadratic(Q, K, V, p: int, normalize: bool = True, scale: float = 1.0):
    """All rows by the definition.  Returns (O [T, v], Z [T]); Z is the sum of the
    scores of each row whether or not it is divided out."""
    T = Q.shape[0]
    O = np.zeros((T, V.shape[1]), dtype=F64)
    Z = np.zeros(T, dtype=F64)
    for i in range(T):
        O[i], Z[i] = fwd_row(Q, K, V, i, p, normalize, scale)
    return O, Z


def _grad_row_terms(G, O, Z, normalize: bool):
    """Upstream gradient with respect to the un-normalised numerator and to the
    denominator:  Ghat_i = G_i / Z_i,  gz_i = -(G_i . O_i)/Z_i  (quotient rule on
    O_i = N_i / Z_i);  un-normalised: Ghat = G, gz = 0."""
    G = np.asarray(G, dtype=F64)
    if not normalize:
        return G.copy(), np.zeros(G.shape[0], dtype=F64)
    Z = np.asarray(Z, dtype=F64)
    Ghat = _safe_div(G, Z[:, None])
    gz = -_safe_div((G * np.asarray(O, dtype=F64)).sum(axis=1), Z)
    return Ghat, gz


def bwd_quadratic(Q, K, V, G, p: int, normalize: bool = True, scale: float = 1.0):
    """Gradient of L = sum_i G_i . O_i with respect to Q, K, V, straight from the
    definition (a t x t score matrix is formed; use on T up to a few thousand)."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    T = Q.shape[0]
    O, Z = fwd_quadratic(Q, K, V, p, normalize, scale)
    Ghat, gz = _grad_row_terms(G, O, Z, normalize)
    mask = np.tril(np.ones((T, T), dtype=F64))
    s = scale * (Q @ K.T)
    a = _ipow(s, p) * mask                              # a_ij, j <= i
    e = (Ghat @ V.T + gz[:, None])                      # dL/da_ij
    t = p * _ipow(s, p - 1) * e * mask                  # dL/ds_ij
    dQ = scale * (t @ K)
    dK = scale * (t.T @ Q)
    dV = a.T @ Ghat
    return dQ, dK, dV


def bwd_dq_row(Q, K, V, G, i: int, p: int, normalize: bool = True, scale: float = 1.0, saved=None):
    """dQ_i alone, O(i d): needs only row i of the forward pass.  saved = (O_i, Z_i): evaluate at these
    saved forward results instead of recomputing them (a backward pass is handed O and Z as inputs; this is
    how a test measures what rounding the saved output to its storage type does to a row)."""
    O_i, Z_i = fwd_row(Q, K, V, i, p, normalize, scale) if saved is None else (np.asarray(saved[0], dtype=F64), float(saved[1]))
    g = np.asarray(G[i], dtype=F64)
    if normalize:
        if Z_i == 0.0:
            return np.zeros(Q.shape[1], dtype=F64)
        ghat = g / Z_i
        gz = -(g @ O_i) / Z_i
    else:
        ghat, gz = g, 0.0
    Kc = np.asarray(K[: i + 1], dtype=F64)
    Vc = np.asarray(V[: i + 1], dtype=F64)
    s = scale * (Kc @ np.asarray(Q[i], dtype=F64))
    t = p * _ipow(s, p - 1) * (Vc @ ghat + gz)
    return scale * (t @ Kc)


def bwd_dkdv_col(Q, K, V, G, O, Z, j: int, p: int, normalize: bool = True, scale: float = 1.0):
    """(dK_j, dV_j) alone, O((T-j) d): needs O and Z of the rows i >= j (pass full
    arrays; they may come from any of this file's forward functions)."""
    Qc = np.asarray(Q[j:], dtype=F64)
    Ghat, gz = _grad_row_terms(G[j:], O[j:], Z[j:], normalize)
    s = scale * (Qc @ np.asarray(K[j], dtype=F64))
    a = _ipow(s, p)
    e = Ghat @ np.asarray(V[j], dtype=F64) + gz
    t = p * _ipow(s, p - 1) * e
    return scale * (t @ Qc), a @ Ghat


# --------------------------------------------------------------------------------------
# Recurrent / chunked form with the explicit SPOW state (Sec. 2 Eq. (6), "Chunked form",
# App. A; update-state / query-state of Sec. 4.1 Eq. (10); gamma / zeta of App. E.2, E.4)
# --------------------------------------------------------------------------------------

def fwd_chunked(Q, K, V, p: int, chunk: int, normalize: bool = True, scale: float = 1.0):
    """Chunked form.  The state entering a chunk holds every strictly earlier chunk,
    S = sum_j phi(k_j) [v_j, 1]^T  (the extra column is the sum of expanded keys, the
    normaliser state gamma of App. E.2); all pairs inside a chunk, diagonal included,
    go through the attention form; the two are combined as in App. E.4:
    (Y_intra + phi(Q) S) / (zeta + phi(Q) gamma).  Any T (last chunk may be short).
    Returns (O, Z)."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    T, d = Q.shape
    v = V.shape[1]
    D = dim_spow(d, p)
    Vp = np.concatenate([V, np.ones((T, 1), dtype=F64)], axis=1)      # [V, 1]
    S = np.zeros((D, v + 1), dtype=F64)
    O = np.zeros((T, v), dtype=F64)
    Z = np.zeros(T, dtype=F64)
    for lo in range(0, T, chunk):
        hi = min(lo + chunk, T)
        Qc, Kc, Vc = Q[lo:hi] * scale, K[lo:hi], Vp[lo:hi]
        inter = spow(Qc, p) @ S                                        # query-state
        m = np.tril(np.ones((hi - lo, hi - lo), dtype=F64))
        intra = (_ipow(Qc @ Kc.T, p) * m) @ Vc                         # attention form
        tot = inter + intra
        Z[lo:hi] = tot[:, v]
        O[lo:hi] = _safe_div(tot[:, :v], tot[:, v:v + 1]) if normalize else tot[:, :v]
        S = S + spow(Kc, p).T @ Vc                                     # update-state
    return O, Z


def fwd_recurrent(Q, K, V, p: int, normalize: bool = True, scale: float = 1.0):
    """Recurrent form, Sec. 2 Eq. (6): S_i = S_{i-1} + phi(K_i) [V_i,1]^T, Y_i = S_i^T phi(Q_i)."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    T, d = Q.shape
    v = V.shape[1]
    S = np.zeros((dim_spow(d, p), v + 1), dtype=F64)
    O = np.zeros((T, v), dtype=F64)
    Z = np.zeros(T, dtype=F64)
    for i in range(T):
        S = S + np.outer(spow(K[i], p), np.append(V[i], 1.0))
        y = spow(scale * Q[i], p) @ S
        Z[i] = y[v]
        O[i] = (y[:v] / y[v] if y[v] != 0.0 else 0.0) if normalize else y[:v]
    return O, Z


def bwd_chunked(Q, K, V, G, p: int, chunk: int, normalize: bool = True, scale: float = 1.0):
    """Backward of the chunked form (derived; the paper has none).

    Forward sweep: with the state S_n entering chunk n,
        d phi(q_i) = S_n ghat'_i,       dq_i += J_phi(q_i)^T d phi(q_i)
    Reverse sweep: R_m = sum over later chunks of phi(q_i) ghat'_i^T  (gradient of the
    loss with respect to the state leaving chunk m),
        dv'_j = R_m^T phi(k_j),         dk_j += J_phi(k_j)^T (R_m v'_j)
    where v' = [v, 1] and ghat' = [G/Z, -(G.O)/Z]; pairs inside a chunk use the
    attention-form gradient.  Returns (dQ, dK, dV)."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    T, d = Q.shape
    v = V.shape[1]
    D = dim_spow(d, p)
    O, Z = fwd_chunked(Q, K, V, p, chunk, normalize, scale)
    Ghat, gz = _grad_row_terms(G, O, Z, normalize)
    Gp = np.concatenate([Ghat, gz[:, None]], axis=1)                   # ghat'
    Vp = np.concatenate([V, np.ones((T, 1), dtype=F64)], axis=1)
    Qs = Q * scale
    dQs = np.zeros((T, d), dtype=F64)
    dK = np.zeros((T, d), dtype=F64)
    dVp = np.zeros((T, v + 1), dtype=F64)
    bounds = [(lo, min(lo + chunk, T)) for lo in range(0, T, chunk)]
    S = np.zeros((D, v + 1), dtype=F64)
    for lo, hi in bounds:
        Qc, Kc, Vc, Gc = Qs[lo:hi], K[lo:hi], Vp[lo:hi], Gp[lo:hi]
        m = np.tril(np.ones((hi - lo, hi - lo), dtype=F64))
        s = Qc @ Kc.T
        e = Gc @ Vc.T
        t = p * _ipow(s, p - 1) * e * m
        dQs[lo:hi] += t @ Kc
        dK[lo:hi] += t.T @ Qc
        dVp[lo:hi] += (_ipow(s, p) * m).T @ Gc
        dQs[lo:hi] += spow_jacobian_transpose_apply(Qc, Gc @ S.T, p)
        S = S + spow(Kc, p).T @ Vc
    R = np.zeros((D, v + 1), dtype=F64)
    for lo, hi in reversed(bounds):
        Qc, Kc, Vc, Gc = Qs[lo:hi], K[lo:hi], Vp[lo:hi], Gp[lo:hi]
        dVp[lo:hi] += spow(Kc, p) @ R
        dK[lo:hi] += spow_jacobian_transpose_apply(Kc, Vc @ R.T, p)
        R = R + spow(Qc, p).T @ Gc
    return dQs * scale, dK, dVp[:, :v]


# --------------------------------------------------------------------------------------
# Gating (Sec. 2 "Gating"; gated update-state of App. E.2, discounted cumulative sum of App. E.3)
#
# The paper adopts a learned gating value per timestep (and per head) and gives the operation
# only at chunk granularity: the state is multiplied by a decay factor before the chunk's update
# is added (App. E.2), and the cumulative sum over chunks discounts by one factor per chunk
# (App. E.3).  The per-timestep definition both come from is the one written out here: with
# log-gates l_t <= 0 and b_i = l_0 + ... + l_i, the pair (i, j), j <= i, carries the product of
# the gates of the steps j+1 .. i,
#       a_ij = s_ij^p * exp(b_i - b_j),        s_ij = scale * (q_i . k_j),
# and everything else (sum, normalisation by the sum of the gated weights) is as before.
# Recurrent form: S_t = g_t S_{t-1} + phi(k_t) [v_t, 1]^T,  y_t = S_t^T phi(q_t).
# --------------------------------------------------------------------------------------

def cum_log_gates(log_g) -> np.ndarray:
    """b_i = sum_{t <= i} log g_t."""
    return np.cumsum(np.asarray(log_g, dtype=F64))


def _gate_matrix(b: np.ndarray) -> np.ndarray:
    """exp(b_i - b_j) for j <= i, 0 above the diagonal."""
    T = b.shape[0]
    diff = b[:, None] - b[None, :]
    mask = np.tril(np.ones((T, T), dtype=bool))
    return np.where(mask, np.exp(np.where(mask, diff, 0.0)), 0.0)


def fwd_quadratic_gated(Q, K, V, log_g, p: int, normalize: bool = True, scale: float = 1.0):
    """All rows by the definition with gating.  Returns (O [T, v], Z [T])."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    a = _ipow(scale * (Q @ K.T), p) * _gate_matrix(cum_log_gates(log_g))
    N = a @ V
    Z = a.sum(axis=1)
    return (_safe_div(N, Z[:, None]) if normalize else N), Z


def fwd_row_gated(Q, K, V, log_g, i: int, p: int, normalize: bool = True, scale: float = 1.0):
    """One output row by the definition with gating: (O_i [v], Z_i)."""
    b = cum_log_gates(log_g[: i + 1])
    q = np.asarray(Q[i], dtype=F64)
    Kc = np.asarray(K[: i + 1], dtype=F64)
    Vc = np.asarray(V[: i + 1], dtype=F64)
    a = _ipow(scale * (Kc @ q), p) * np.exp(b[i] - b)
    N = a @ Vc
    Z = a.sum()
    if normalize:
        return (N / Z if Z != 0.0 else np.zeros_like(N)), Z
    return N, Z


def bwd_quadratic_gated(Q, K, V, log_g, G, p: int, normalize: bool = True, scale: float = 1.0):
    """Gradient of L = sum_i G_i . O_i with respect to Q, K, V and the log-gates, straight from
    the definition.  With e_ij = dL/da_ij:  a_ij depends on b_i with derivative a_ij and on b_j
    with derivative -a_ij, so  dL/db_i = sum_{j<=i} e_ij a_ij - sum_{i'>=i} e_i'i a_i'i,  and
    b_i = sum_{t<=i} l_t gives  dL/dl_t = sum_{i>=t} dL/db_i.  Returns (dQ, dK, dV, dlog_g)."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    O, Z = fwd_quadratic_gated(Q, K, V, log_g, p, normalize, scale)
    Ghat, gz = _grad_row_terms(G, O, Z, normalize)
    gate = _gate_matrix(cum_log_gates(log_g))
    s = scale * (Q @ K.T)
    a = _ipow(s, p) * gate                               # a_ij, j <= i
    e = Ghat @ V.T + gz[:, None]                         # dL/da_ij
    t = p * _ipow(s, p - 1) * gate * e                   # dL/ds_ij
    dQ = scale * (t @ K)
    dK = scale * (t.T @ Q)
    dV = a.T @ Ghat
    ea = e * a
    db = ea.sum(axis=1) - ea.sum(axis=0)
    dlog_g = np.cumsum(db[::-1])[::-1].copy()
    return dQ, dK, dV, dlog_g


def fwd_recurrent_gated(Q, K, V, log_g, p: int, normalize: bool = True, scale: float = 1.0):
    """Gated recurrent form: S_t = g_t S_{t-1} + phi(k_t) [v_t, 1]^T,  y_t = S_t^T phi(scale q_t)."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    g = np.exp(np.asarray(log_g, dtype=F64))
    T, d = Q.shape
    v = V.shape[1]
    S = np.zeros((dim_spow(d, p), v + 1), dtype=F64)
    O = np.zeros((T, v), dtype=F64)
    Z = np.zeros(T, dtype=F64)
    for i in range(T):
        S = g[i] * S + np.outer(spow(K[i], p), np.append(V[i], 1.0))
        y = spow(scale * Q[i], p) @ S
        Z[i] = y[v]
        O[i] = (y[:v] / y[v] if y[v] != 0.0 else 0.0) if normalize else y[:v]
    return O, Z


# --------------------------------------------------------------------------------------
# Single-token decode step (Sec. 2 Eq. (6), one iteration; the inference use of App. D)
# --------------------------------------------------------------------------------------

def decode_state_init(d: int, v: int, p: int) -> np.ndarray:
    """The empty state: D x (v + 1) zeros, D = C(d + p - 1, p); column v is the normaliser."""
    return np.zeros((dim_spow(d, p), v + 1), dtype=F64)


def decode_step(S, q, k, v, p: int, normalize: bool = True, scale: float = 1.0, log_g=None):
    """One token: S' = g S + phi(k) [v, 1]^T, then y = S'^T phi(scale q) (the token attends to
    itself).  Returns (S', o [v], z); g = exp(log_g), 1 when log_g is None."""
    S = np.asarray(S, dtype=F64)
    vv = np.asarray(v, dtype=F64)
    g = 1.0 if log_g is None else math.exp(float(log_g))
    S_new = g * S + np.outer(spow(np.asarray(k, dtype=F64), p), np.append(vv, 1.0))
    y = spow(scale * np.asarray(q, dtype=F64), p) @ S_new
    z = y[-1]
    if normalize:
        o = y[:-1] / z if z != 0.0 else np.zeros_like(vv)
    else:
        o = y[:-1]
    return S_new, o, z


def _chunk_gate_factors(b: np.ndarray, lo: int, hi: int):
    """For the chunk [lo, hi): the decay of each query since the chunk's start, exp(b_i - B),
    B = b_{lo-1} (0 for the first chunk); of each key until the chunk's end, exp(b_{hi-1} - b_j);
    and across the whole chunk, exp(b_{hi-1} - B).  All are <= 1 for log-gates <= 0."""
    B = b[lo - 1] if lo > 0 else 0.0
    return np.exp(b[lo:hi] - B), np.exp(b[hi - 1] - b[lo:hi]), math.exp(b[hi - 1] - B)


def fwd_chunked_gated(Q, K, V, log_g, p: int, chunk: int, normalize: bool = True, scale: float = 1.0):
    """Chunked form with gating: the state entering a chunk is the gated sum of all earlier
    keys as seen from the chunk's start; a query i of the chunk sees it decayed by
    exp(b_i - B); the chunk's update weighs key j by its decay until the chunk's end, and the
    state is multiplied by the decay across the chunk before the update is added (App. E.2,
    E.3).  Pairs inside a chunk use the attention form with exp(b_i - b_j).  Returns (O, Z)."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    T, d = Q.shape
    v = V.shape[1]
    b = cum_log_gates(log_g)
    Vp = np.concatenate([V, np.ones((T, 1), dtype=F64)], axis=1)
    S = np.zeros((dim_spow(d, p), v + 1), dtype=F64)
    O = np.zeros((T, v), dtype=F64)
    Z = np.zeros(T, dtype=F64)
    for lo in range(0, T, chunk):
        hi = min(lo + chunk, T)
        qf, kf, lam = _chunk_gate_factors(b, lo, hi)
        Qc, Kc, Vc = Q[lo:hi] * scale, K[lo:hi], Vp[lo:hi]
        inter = qf[:, None] * (spow(Qc, p) @ S)
        intra = (_ipow(Qc @ Kc.T, p) * _gate_matrix(b[lo:hi])) @ Vc
        tot = inter + intra
        Z[lo:hi] = tot[:, v]
        O[lo:hi] = _safe_div(tot[:, :v], tot[:, v:v + 1]) if normalize else tot[:, :v]
        S = lam * S + spow(Kc, p).T @ (kf[:, None] * Vc)
    return O, Z


def bwd_chunked_gated(Q, K, V, log_g, G, p: int, chunk: int, normalize: bool = True, scale: float = 1.0):
    """Backward of the gated chunked form (derived).  Mirrors bwd_chunked with the factors of
    fwd_chunked_gated; the reverse sweep carries R_m, the gradient with respect to the state
    leaving chunk m, discounted the same way.  The gradient of the log-gates is assembled from
    the row and column sums of e_ij a_ij, which the sweeps provide as
    q_i . dq_i / p  and  k_j . dk_j / p  (a_ij is homogeneous of degree p in q_i and in k_j).
    Returns (dQ, dK, dV, dlog_g)."""
    Q = np.asarray(Q, dtype=F64); K = np.asarray(K, dtype=F64); V = np.asarray(V, dtype=F64)
    T, d = Q.shape
    v = V.shape[1]
    D = dim_spow(d, p)
    b = cum_log_gates(log_g)
    O, Z = fwd_chunked_gated(Q, K, V, log_g, p, chunk, normalize, scale)
    Ghat, gz = _grad_row_terms(G, O, Z, normalize)
    Gp = np.concatenate([Ghat, gz[:, None]], axis=1)
    Vp = np.concatenate([V, np.ones((T, 1), dtype=F64)], axis=1)
    Qs = Q * scale
    dQs = np.zeros((T, d), dtype=F64)
    dK = np.zeros((T, d), dtype=F64)
    dVp = np.zeros((T, v + 1), dtype=F64)
    bounds = [(lo, min(lo + chunk, T)) for lo in range(0, T, chunk)]
    S = np.zeros((D, v + 1), dtype=F64)
    for lo, hi in bounds:
        qf, kf, lam = _chunk_gate_factors(b, lo, hi)
        Qc, Kc, Vc, Gc = Qs[lo:hi], K[lo:hi], Vp[lo:hi], Gp[lo:hi]
        gate = _gate_matrix(b[lo:hi])
        s = Qc @ Kc.T
        e = Gc @ Vc.T
        t = p * _ipow(s, p - 1) * gate * e
        dQs[lo:hi] += t @ Kc
        dK[lo:hi] += t.T @ Qc
        dVp[lo:hi] += (_ipow(s, p) * gate).T @ Gc
        dQs[lo:hi] += qf[:, None] * spow_jacobian_transpose_apply(Qc, Gc @ S.T, p)
        S = lam * S + spow(Kc, p).T @ (kf[:, None] * Vc)
    R = np.zeros((D, v + 1), dtype=F64)
    for lo, hi in reversed(bounds):
        qf, kf, lam = _chunk_gate_factors(b, lo, hi)
        Qc, Kc, Vc, Gc = Qs[lo:hi], K[lo:hi], Vp[lo:hi], Gp[lo:hi]
        dVp[lo:hi] += kf[:, None] * (spow(Kc, p) @ R)
        dK[lo:hi] += kf[:, None] * spow_jacobian_transpose_apply(Kc, Vc @ R.T, p)
        R = lam * R + spow(Qc, p).T @ (qf[:, None] * Gc)
    db = ((Qs * dQs).sum(axis=1) - (K * dK).sum(axis=1)) / p
    dlog_g = np.cumsum(db[::-1])[::-1].copy()
    return dQs * scale, dK, dVp[:, :v], dlog_g


# --------------------------------------------------------------------------------------
# [B, H, T, d] wrappers
# --------------------------------------------------------------------------------------

def fwd_bhtd(Q, K, V, p, chunk=None, normalize=True, scale=1.0, log_g=None):
    """Forward on [B,H,T,d] arrays; ``chunk=None`` uses the attention form; ``log_g`` [B,H,T]
    switches gating on."""
    B, H, T, _ = Q.shape
    O = np.zeros(V.shape, dtype=F64)
    Z = np.zeros((B, H, T), dtype=F64)
    for b in range(B):
        for h in range(H):
            if log_g is not None:
                if chunk is None:
                    O[b, h], Z[b, h] = fwd_quadratic_gated(Q[b, h], K[b, h], V[b, h], log_g[b, h], p, normalize, scale)
                else:
                    O[b, h], Z[b, h] = fwd_chunked_gated(Q[b, h], K[b, h], V[b, h], log_g[b, h], p, chunk, normalize, scale)
            elif chunk is None:
                O[b, h], Z[b, h] = fwd_quadratic(Q[b, h], K[b, h], V[b, h], p, normalize, scale)
            else:
                O[b, h], Z[b, h] = fwd_chunked(Q[b, h], K[b, h], V[b, h], p, chunk, normalize, scale)
    return O, Z


def bwd_bhtd(Q, K, V, G, p, chunk=None, normalize=True, scale=1.0, log_g=None):
    """Backward on [B,H,T,d] arrays; ``chunk=None`` uses the attention form.  With ``log_g``
    [B,H,T] returns (dQ, dK, dV, dlog_g), else (dQ, dK, dV)."""
    B, H = Q.shape[:2]
    dQ = np.zeros(Q.shape, dtype=F64); dK = np.zeros(K.shape, dtype=F64); dV = np.zeros(V.shape, dtype=F64)
    if log_g is not None:
        dL = np.zeros(log_g.shape, dtype=F64)
        for b in range(B):
            for h in range(H):
                if chunk is None:
                    r = bwd_quadratic_gated(Q[b, h], K[b, h], V[b, h], log_g[b, h], G[b, h], p, normalize, scale)
                else:
                    r = bwd_chunked_gated(Q[b, h], K[b, h], V[b, h], log_g[b, h], G[b, h], p, chunk, normalize, scale)
                dQ[b, h], dK[b, h], dV[b, h], dL[b, h] = r
        return dQ, dK, dV, dL
    for b in range(B):
        for h in range(H):
            if chunk is None:
                r = bwd_quadratic(Q[b, h], K[b, h], V[b, h], G[b, h], p, normalize, scale)
            else:
                r = bwd_chunked(Q[b, h], K[b, h], V[b, h], G[b, h], p, chunk, normalize, scale)
            dQ[b, h], dK[b, h], dV[b, h] = r
    return dQ, dK, dV
