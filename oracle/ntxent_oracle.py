"""Plain float64 NumPy oracle of the decomposed self-supervised contrastive loss (test infrastructure,
never on the product path).

The paper states (Sec. 4.1, last sentence; Conclusion) that the same decomposition applies to the contrastive
loss of self-supervised learning (SimCLR, MoCo-v3) and prints no formula for it.  Reading taken here: SimCLR's
normalised-temperature cross-entropy.  Z (B x d, B = 2M) holds the features of two views of M samples, view
one in rows 0..M-1 and view two in rows M..2M-1, so the positive of row i is row p(i) = (i + M) mod B; a row
is never its own negative (the self-similarity is left out of the softmax):

    l_i = log sum_{k != i} exp(s <z_i, z_k>)  -  s <z_i, z_p(i)>          L = (1/B) sum_i l_i

Decomposition as in Sec. 4.1: rank r of N owns the rows R_r = [r*b, (r+1)*b), b = B/N, forms only its b x B
block of logits s Z_r Z^T, and its outputs carry the factor 1/B, so the SUM over ranks equals the full loss
and gradients.  With P the row softmax over k != i and G_ik = P_ik - [k = p(i)] (G_ii = 0):

    loss_r = (1/B) sum_{i in R_r} l_i
    gZ_r   = (s/B) [ rows i in R_r:  sum_k G_ik z_k      (query side, lands in the rank's own rows)
                   + every row k:    sum_{i in R_r} G_ik z_i ]   (key side: what Eq. 5 / Eq. 7 send to other ranks)
    gs_r   = (1/B) sum_{i in R_r} sum_k G_ik <z_i, z_k>
Gradients are with respect to Z as given and to the multiplier s itself.
"""
from __future__ import annotations

import numpy as np

_CHUNK = 2048


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _rows_terms(Z: np.ndarray, s: float, rows: np.ndarray, magnitudes: bool = False):
    """Sums over the query rows `rows`, WITHOUT the 1/B factor: (sum of l_i, query-side gradient rows, key-side
    gradient B x d, derivative w.r.t. s).  With magnitudes=True every term enters by its absolute value (the scale
    of the elementwise parity bound) and the first entry is None."""
    B, d = Z.shape
    M = B // 2
    ce_sum, dS = 0.0, 0.0
    dq = np.zeros((rows.size, d))
    dk = np.zeros((B, d))
    for lo in range(0, rows.size, _CHUNK):
        idx = rows[lo:lo + _CHUNK]
        k = np.arange(idx.size)
        Zc = Z[idx]
        cos = Zc @ Z.T
        logits = s * cos
        logits[k, idx] = -np.inf                          # a row is not its own negative
        m = logits.max(axis=1)
        lse = m + np.log(np.exp(logits - m[:, None]).sum(axis=1))
        pos = (idx + M) % B
        G = np.exp(logits - lse[:, None])                 # softmax over k != i (exp(-inf) = 0 on the diagonal)
        G[k, pos] -= 1.0
        if magnitudes:
            G = np.abs(G)
            dq[lo:lo + idx.size] = abs(s) * (G @ np.abs(Z))
            dk += abs(s) * (G.T @ np.abs(Zc))
            dS += float(np.sum(G * np.abs(cos)))
        else:
            ce_sum += float(np.sum(lse - s * cos[k, pos]))
            dq[lo:lo + idx.size] = s * (G @ Z)
            dk += s * (G.T @ Zc)
            dS += float(np.sum(G * cos))
    return (None if magnitudes else ce_sum), dq, dk, dS


def ntxent_rank(Z, s: float, rank: int, N: int):
    """(loss_r, gZ_r (B x d), gs_r) of rank `rank` of N, each carrying 1/B."""
    Z = _f64(Z)
    B = Z.shape[0]
    if B % 2 or N <= 0 or B % N or not (0 <= rank < N):
        raise ValueError("need an even number of rows, B % N == 0 and 0 <= rank < N")
    b = B // N
    R = np.arange(rank * b, (rank + 1) * b)
    ce, dq, dk, dS = _rows_terms(Z, s, R)
    g = dk / B
    g[R] += dq / B
    return ce / B, g, dS / B


def ntxent_full(Z, s: float):
    """The non-decomposed loss: (L, dL/dZ, dL/ds)."""
    return ntxent_rank(Z, s, 0, 1)


def ntxent_rank_term_scale(Z, s: float, rank: int, N: int):
    """(scale of gZ_r entries (B x d), scale of gs_r): ntxent_rank's sums with every term's magnitude."""
    Z = _f64(Z)
    B = Z.shape[0]
    b = B // N
    R = np.arange(rank * b, (rank + 1) * b)
    _, aq, ak, aS = _rows_terms(Z, s, R, magnitudes=True)
    a = ak / B
    a[R] += aq / B
    return a, aS / B
