"""Plain fp64 causal softmax attention: the definition the method must reproduce.

TEST INFRASTRUCTURE ONLY (see the package docstring).  numpy, fp64, no tiling of
the key axis, no online softmax, no reordering: every query row sees its whole
key range at once, exactly as Eq. 1 of Section 3.1 of the DistFlashAttn paper
writes it (softmax(q [k_1..k_p]^T / sqrt(d)) [v_1..v_p], token-level causal).
The paper states the method is exact attention (Sections 1 and 3), so this
definition *is* the expected result of the chunked / merged / balanced path.

Conventions
-----------
* Q, dO, O, dQ: float64 arrays [H_q, N, d];  K, V, dK, dV: [H_kv, N, d].
* Grouped-query attention (Section 4, "model setup"): H_kv key/value heads, each
  shared by g = H_q / H_kv consecutive query heads: query head h uses kv head
  h // g.  Gradients of a kv head sum over its g query heads.
* `scale` multiplies q.k before the softmax (Eq. 1 uses 1/sqrt(d)).
* The causal mask keeps key j for query i iff j <= i (a token attends to itself
  and to earlier tokens; Section 3.2).
* L is the natural-log logsumexp of the scaled, masked scores, L = m + log(l)
  in the notation of the appendix's forward pseudo-code.
* "Pair (p, r)" = query chunk p (rows [pC, (p+1)C)) against key/value chunk r
  (columns [rC, (r+1)C)), r <= p.  r == p is the causal diagonal chunk.

Functions with no external pin would say "parity unpinned" here; every function
below is pinned by tests/test_oracle_*.py (finite differences, library softmax,
closed forms, invariants, merge == monolithic).
"""
from __future__ import annotations

import numpy as np


def _kv_head(h: int, h_q: int, h_kv: int) -> int:
    assert h_q % h_kv == 0
    return h // (h_q // h_kv)


def _scores(q_rows: np.ndarray, k: np.ndarray, scale: float, row0: int,
            causal: bool, col0: int = 0) -> np.ndarray:
    """scale * q k^T with -inf where the key index exceeds the query index.

    q_rows are global rows row0.. ; k columns are global columns col0.. .
    """
    s = scale * (q_rows @ k.T)
    if causal:
        i = row0 + np.arange(q_rows.shape[0])[:, None]
        j = col0 + np.arange(k.shape[0])[None, :]
        s = np.where(j <= i, s, -np.inf)
    return s


def attention_fwd(Q, K, V, scale, causal=True, row_block=512):
    """Monolithic forward over the whole sequence (Eq. 1, Section 3.1).

    Returns (O [H_q,N,d], L [H_q,N]).  Rows are processed in blocks only to bound
    memory; each row still sees every key at once.
    """
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    h_q, n, d = Q.shape
    h_kv = K.shape[0]
    O = np.empty((h_q, n, V.shape[2]), np.float64)
    L = np.empty((h_q, n), np.float64)
    for h in range(h_q):
        kh = _kv_head(h, h_q, h_kv)
        for r0 in range(0, n, row_block):
            r1 = min(n, r0 + row_block)
            ncols = r1 if causal else K.shape[1]
            s = _scores(Q[h, r0:r1], K[kh, :ncols], scale, r0, causal)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            l = e.sum(axis=1, keepdims=True)
            O[h, r0:r1] = (e / l) @ V[kh, :ncols]
            L[h, r0:r1] = (m + np.log(l))[:, 0]
    return O, L


def softmax_weights(Q, K, scale, causal=True):
    """The full matrix P = softmax(scale QK^T + mask) per query head (small inputs only)."""
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64)
    h_q, n, _ = Q.shape
    h_kv = K.shape[0]
    P = np.empty((h_q, n, K.shape[1]), np.float64)
    for h in range(h_q):
        s = _scores(Q[h], K[_kv_head(h, h_q, h_kv)], scale, 0, causal)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        P[h] = e / e.sum(axis=1, keepdims=True)
    return P


def attention_bwd(Q, K, V, dO, scale, causal=True, row_block=512):
    """Analytic backward of the monolithic forward.

    With P the softmax weights: dV = P^T dO; dP = dO V^T; D_i = sum_j P_ij dP_ij;
    dS = P o (dP - D); dQ = scale dS K; dK = scale dS^T Q.  Returns (dQ, dK, dV).
    """
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64); dO = np.asarray(dO, np.float64)
    h_q, n, d = Q.shape
    h_kv = K.shape[0]
    dQ = np.zeros_like(Q); dK = np.zeros_like(K); dV = np.zeros_like(V)
    for h in range(h_q):
        kh = _kv_head(h, h_q, h_kv)
        for r0 in range(0, n, row_block):
            r1 = min(n, r0 + row_block)
            ncols = r1 if causal else K.shape[1]
            s = _scores(Q[h, r0:r1], K[kh, :ncols], scale, r0, causal)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            p = e / e.sum(axis=1, keepdims=True)
            dp = dO[h, r0:r1] @ V[kh, :ncols].T
            dd = (p * dp).sum(axis=1, keepdims=True)
            ds = p * (dp - dd)
            dV[kh, :ncols] += p.T @ dO[h, r0:r1]
            dQ[h, r0:r1] = scale * (ds @ K[kh, :ncols])
            dK[kh, :ncols] += scale * (ds.T @ Q[h, r0:r1])
    return dQ, dK, dV


def _window_scores(q, k, scale, c, window_chunks):
    """scale * q k^T over a whole head with -inf outside the chunk-level causal window: key j is
    kept for query i iff j <= i and chunk(j) >= chunk(i) - window_chunks, chunk(x) = x // c."""
    n = q.shape[0]
    i = np.arange(n)[:, None]
    j = np.arange(k.shape[0])[None, :]
    keep = (j <= i) & (j // c >= i // c - window_chunks)
    return np.where(keep, scale * (q @ k.T), -np.inf)


def window_attention_fwd(Q, K, V, scale, c, window_chunks):
    """Causal attention local to the query's own chunk of c tokens and the `window_chunks`
    chunks before it (appendix on sparse patterns, local sliding windows, at the granularity the
    paper describes: whole chunks of the preceding workers).  Monolithic per head; returns (O, L)."""
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    h_q, n, _ = Q.shape
    h_kv = K.shape[0]
    O = np.empty((h_q, n, V.shape[2]), np.float64)
    L = np.empty((h_q, n), np.float64)
    for h in range(h_q):
        kh = _kv_head(h, h_q, h_kv)
        s = _window_scores(Q[h], K[kh], scale, c, window_chunks)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=1, keepdims=True)
        O[h] = (e / l) @ V[kh]
        L[h] = (m + np.log(l))[:, 0]
    return O, L


def window_attention_bwd(Q, K, V, dO, scale, c, window_chunks):
    """Analytic backward of window_attention_fwd (same formulas as attention_bwd)."""
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64); dO = np.asarray(dO, np.float64)
    h_q = Q.shape[0]
    h_kv = K.shape[0]
    dQ = np.zeros_like(Q); dK = np.zeros_like(K); dV = np.zeros_like(V)
    for h in range(h_q):
        kh = _kv_head(h, h_q, h_kv)
        s = _window_scores(Q[h], K[kh], scale, c, window_chunks)
        e = np.exp(s - s.max(axis=1, keepdims=True))
        p = e / e.sum(axis=1, keepdims=True)
        dp = dO[h] @ V[kh].T
        ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
        dV[kh] += p.T @ dO[h]
        dQ[h] = scale * (ds @ K[kh])
        dK[kh] += scale * (ds.T @ Q[h])
    return dQ, dK, dV


def delta_rows(O, dO):
    """D_i = sum_c dO_ic O_ic, which equals sum_j P_ij dP_ij for the exact O."""
    return (np.asarray(O, np.float64) * np.asarray(dO, np.float64)).sum(axis=-1)


def pair_fwd(Q, K, V, scale, p, r, c):
    """Partial result of query chunk p against key/value chunk r alone.

    lse_part_i = log sum_{j in chunk r, j<=i} exp(S_ij);  o_part_i = softmax over
    those keys only, times V.  This is what one attn(q_p, k_r, v_r, o^0, s^0) call
    of the balanced algorithm (Appendix A) yields when started from the empty
    state, expressed as normalised output + logsumexp.
    Returns (o_part [H_q,c,d], lse_part [H_q,c]).
    """
    assert r <= p
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    h_q = Q.shape[0]; h_kv = K.shape[0]
    o = np.empty((h_q, c, V.shape[2]), np.float64)
    lse = np.empty((h_q, c), np.float64)
    for h in range(h_q):
        kh = _kv_head(h, h_q, h_kv)
        s = _scores(Q[h, p * c:(p + 1) * c], K[kh, r * c:(r + 1) * c], scale,
                    p * c, causal=True, col0=r * c)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=1, keepdims=True)
        o[h] = (e / l) @ V[kh, r * c:(r + 1) * c]
        lse[h] = (m + np.log(l))[:, 0]
    return o, lse


def pair_bwd(Q, K, V, dO, L, D, scale, p, r, c):
    """Gradient contributions of pair (p, r), using the GLOBAL logsumexp L and D.

    P_ij = exp(S_ij - L_i) is a slice of the monolithic softmax matrix, so summing
    these partials over all pairs gives the monolithic gradients (Section 3.3: the
    backward reuses the saved output / logsumexp and never re-runs the forward).
    Returns (dq_part [H_q,c,d], dk_part [H_kv,c,d], dv_part [H_kv,c,d]).
    """
    assert r <= p
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64); dO = np.asarray(dO, np.float64)
    h_q = Q.shape[0]; h_kv = K.shape[0]
    rows = slice(p * c, (p + 1) * c); cols = slice(r * c, (r + 1) * c)
    dq = np.empty((h_q, c, Q.shape[2]), np.float64)
    dk = np.zeros((h_kv, c, K.shape[2]), np.float64)
    dv = np.zeros((h_kv, c, V.shape[2]), np.float64)
    for h in range(h_q):
        kh = _kv_head(h, h_q, h_kv)
        s = _scores(Q[h, rows], K[kh, cols], scale, p * c, causal=True, col0=r * c)
        pm = np.exp(s - L[h, rows][:, None])
        dp = dO[h, rows] @ V[kh, cols].T
        ds = pm * (dp - D[h, rows][:, None])
        dq[h] = scale * (ds @ K[kh, cols])
        dk[kh] += scale * (ds.T @ Q[h, rows])
        dv[kh] += pm.T @ dO[h, rows]
    return dq, dk, dv


def merge(o_a, lse_a, o_b, lse_b):
    """Exact combination of two partial results for the same queries.

    The rescale(.) step of the balanced algorithm (Section 3.2): with normalised
    partial outputs and their logsumexps, lse = log(e^lse_a + e^lse_b) and
    o = e^(lse_a - lse) o_a + e^(lse_b - lse) o_b.  (0, -inf) is the identity.
    """
    o_a = np.asarray(o_a, np.float64); o_b = np.asarray(o_b, np.float64)
    lse_a = np.asarray(lse_a, np.float64); lse_b = np.asarray(lse_b, np.float64)
    lse = np.logaddexp(lse_a, lse_b)
    with np.errstate(invalid="ignore"):
        wa = np.where(np.isneginf(lse_a), 0.0, np.exp(lse_a - lse))
        wb = np.where(np.isneginf(lse_b), 0.0, np.exp(lse_b - lse))
    return wa[..., None] * o_a + wb[..., None] * o_b, lse


# ---------------------------------------------------------------------------
# Row / column samplers: the same definition evaluated for a few rows (or key
# columns) of one head, for sequences too long to evaluate in full.
# ---------------------------------------------------------------------------

def rows_fwd(q_rows, row_idx, K, V, scale, col_lo=0, col_hi=None):
    """O_i and L_i for the given global query rows of one head.

    q_rows [n_rows,d]; row_idx their global token indices; K, V [n_keys,d] hold
    global key columns col_lo..col_hi-1.  Keys j > i are masked.
    """
    q_rows = np.asarray(q_rows, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    if col_hi is None:
        col_hi = col_lo + K.shape[0]
    s = scale * (q_rows @ K.T)
    j = col_lo + np.arange(K.shape[0])[None, :]
    s = np.where(j <= np.asarray(row_idx)[:, None], s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    return (e / l) @ V, (m + np.log(l))[:, 0]


def rows_dq(q_rows, row_idx, do_rows, l_rows, d_rows, K, V, scale, col_lo=0):
    """dq contribution to the given query rows from key columns col_lo.. (one head),
    given those rows' global logsumexp and D."""
    q_rows = np.asarray(q_rows, np.float64); do_rows = np.asarray(do_rows, np.float64)
    K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    s = scale * (q_rows @ K.T)
    j = col_lo + np.arange(K.shape[0])[None, :]
    s = np.where(j <= np.asarray(row_idx)[:, None], s, -np.inf)
    p = np.exp(s - np.asarray(l_rows, np.float64)[:, None])
    ds = p * (do_rows @ V.T - np.asarray(d_rows, np.float64)[:, None])
    return scale * (ds @ K)


def cols_dkdv(k_cols, v_cols, col_idx, Qh, dOh, Lh, Dh, scale, row_lo=0):
    """dk_j and dv_j for the given global key columns of one kv head, summed over the
    query rows Qh (global rows row_lo..), which may stack several query heads of the
    group one after another only if called once per head and added by the caller.

    Qh, dOh [n_rows,d]; Lh, Dh [n_rows] are those rows' global logsumexp and D.
    """
    k_cols = np.asarray(k_cols, np.float64); v_cols = np.asarray(v_cols, np.float64)
    Qh = np.asarray(Qh, np.float64); dOh = np.asarray(dOh, np.float64)
    s = scale * (Qh @ k_cols.T)
    i = row_lo + np.arange(Qh.shape[0])[:, None]
    s = np.where(np.asarray(col_idx)[None, :] <= i, s, -np.inf)
    p = np.exp(s - np.asarray(Lh, np.float64)[:, None])
    ds = p * (dOh @ v_cols.T - np.asarray(Dh, np.float64)[:, None])
    return scale * (ds.T @ Qh), p.T @ dOh
