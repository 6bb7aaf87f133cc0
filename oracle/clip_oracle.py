"""Plain float64 NumPy oracle (test infrastructure, never on the product path).

Notation follows the paper (Sec. 2.1, Sec. 4.1): B pairs in the global batch, N
ranks, b = B/N pairs per rank, d the feature width, I and T the gathered image
and text features (B x d), s the logit multiplier (the paper's `t` in Alg. 1,
which multiplies the dot products).  Rank r (0-based, as Alg. 1's `rank`) owns
the global rows R_r = [r*b, (r+1)*b).

Conventions (readings where the paper leaves a choice):
  * Normalisation: Alg. 1 takes the mean cross-entropy over the rank's b rows,
    halves the sum of the two directions and averages over the N ranks.  That
    composes to  L = (1/(2B)) * sum_i (ce1_i + ce2_i).  Per-rank results here
    carry the global factor c = 1/(2B), so the SUM over ranks of the per-rank
    outputs equals the full result (Eq. 3-5, 7).
  * Gradients are with respect to the arrays as given (no projection through
    an L2 normalisation) and with respect to the multiplier s itself.

DisCo is exact (Sec. 4.1, Eq. 3), so the oracle is the plain definition of
the original loss (Eq. 1) written out, plus the same sums restricted to one
rank's rows (Eq. 4-6).  Row chunking below only bounds memory; each chunk is
the definition applied to those rows.
"""
from __future__ import annotations

import numpy as np

_CHUNK = 2048


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _row_logsumexp(Z: np.ndarray) -> np.ndarray:
    """log sum_j exp(Z_ij) per row, by max subtraction."""
    m = Z.max(axis=1)
    return m + np.log(np.exp(Z - m[:, None]).sum(axis=1))


def directional_terms(X: np.ndarray, Y: np.ndarray, s: float, rows: np.ndarray):
    """One direction of Eq. 1 restricted to the query rows `rows`.

    For each i in rows:  ce_i = logsumexp_j(s <X_i, Y_j>) - s <X_i, Y_i>,
    i.e. Alg. 1's cross_entropy(logits, labels) with the positive on the global
    diagonal.  Returns, WITHOUT the 1/(2B) factor,
      ce_sum = sum_i ce_i
      dXq    = sum_j (P_ij - [j = i]) * s * Y_j            (len(rows) x d), query-side gradient
      dY     = sum_i (P_ij - [j = i]) * s * X_i            (B x d), key-side gradient
      dS     = sum_ij (P_ij - [j = i]) * <X_i, Y_j>        derivative w.r.t. s
    with P = row softmax of the logits.
    """
    X, Y = _f64(X), _f64(Y)
    B, d = Y.shape
    rows = np.asarray(rows, dtype=np.int64)
    ce_sum, dS = 0.0, 0.0
    dXq = np.zeros((rows.size, d))
    dY = np.zeros((B, d))
    for lo in range(0, rows.size, _CHUNK):
        idx = rows[lo:lo + _CHUNK]
        Xc = X[idx]
        cos = Xc @ Y.T                                   # raw similarities, chunk x B
        Z = s * cos                                      # logits (Alg. 1: dot(...) * t)
        lse = _row_logsumexp(Z)
        k = np.arange(idx.size)
        ce_sum += float(np.sum(lse - Z[k, idx]))
        G = np.exp(Z - lse[:, None])                     # softmax rows
        G[k, idx] -= 1.0                                 # minus one-hot of the label column
        dXq[lo:lo + idx.size] = s * (G @ Y)
        dY += s * (G.T @ Xc)
        dS += float(np.sum(G * cos))
    return ce_sum, dXq, dY, dS


def directional_term_scale(X: np.ndarray, Y: np.ndarray, s: float, rows: np.ndarray):
    """Sum of the magnitudes of the terms that directional_terms adds up.

    aXq[i] = sum_j |P_ij - [j = i]| * |s| * |Y_j|   and   aY[j] = sum_i |P_ij - [j = i]| * |s| * |X_i|
    (elementwise absolute values).  An implementation that rounds each factor of every product
    to a format with unit roundoff u errs by at most about 2u times this, whatever cancels in the
    sum itself; the parity tests use it as the scale of their elementwise bound.
    """
    X, Y = _f64(X), _f64(Y)
    B, d = Y.shape
    rows = np.asarray(rows, dtype=np.int64)
    aXq = np.zeros((rows.size, d))
    aY = np.zeros((B, d))
    absY = np.abs(Y)
    for lo in range(0, rows.size, _CHUNK):
        idx = rows[lo:lo + _CHUNK]
        Xc = X[idx]
        Z = s * (Xc @ Y.T)
        G = np.exp(Z - _row_logsumexp(Z)[:, None])
        G[np.arange(idx.size), idx] -= 1.0
        G = np.abs(G)
        aXq[lo:lo + idx.size] = abs(s) * (G @ absY)
        aY += abs(s) * (G.T @ np.abs(Xc))
    return aXq, aY


def disco_rank_term_scale(I, T, s: float, rank: int, N: int):
    """Elementwise scale (B x d each) for gI_r and gT_r of disco_rank: same sums with every term's magnitude."""
    I, T = _f64(I), _f64(T)
    B = I.shape[0]
    b = B // N
    c = 1.0 / (2.0 * B)
    R = np.arange(rank * b, (rank + 1) * b)
    aI_q, aT_k = directional_term_scale(I, T, s, R)
    aT_q, aI_k = directional_term_scale(T, I, s, R)
    sI = c * aI_k
    sI[R] += c * aI_q
    sT = c * aT_k
    sT[R] += c * aT_q
    return sI, sT


def disco_rank_gs_term_scale(I, T, s: float, rank: int, N: int) -> float:
    """Scale for gs_r of disco_rank: c * sum over both blocks of |P_ij - [j = i]| * |<x_i, y_j>|.

    The derivative w.r.t. s adds up (P_ij - [j = i]) <x_i, y_j> over all pairs of both blocks; this is the same sum
    with every term's magnitude, the bound that a rounding of each P_ij moves gs_r by at most u times.
    """
    I, T = _f64(I), _f64(T)
    B = I.shape[0]
    b = B // N
    R = np.arange(rank * b, (rank + 1) * b)
    total = 0.0
    for X, Y in ((I, T), (T, I)):
        for lo in range(0, b, _CHUNK):
            idx = R[lo:lo + _CHUNK]
            cos = X[idx] @ Y.T
            Z = s * cos
            G = np.exp(Z - _row_logsumexp(Z)[:, None])
            G[np.arange(idx.size), idx] -= 1.0
            total += float(np.sum(np.abs(G) * np.abs(cos)))
    return total / (2.0 * B)


def clip_loss_full(I, T, s: float):
    """Original, non-distributed CLIP loss (Eq. 1) and its gradients.

    L = (1/(2B)) [ sum_i CE(row i of s I T^T, i) + sum_i CE(row i of s T I^T, i) ].
    Returns (L, dL/dI, dL/dT, dL/ds).
    """
    I, T = _f64(I), _f64(T)
    B = I.shape[0]
    c = 1.0 / (2.0 * B)
    allrows = np.arange(B)
    ce1, dI_q, dT_k, ds1 = directional_terms(I, T, s, allrows)   # image -> text
    ce2, dT_q, dI_k, ds2 = directional_terms(T, I, s, allrows)   # text -> image
    return c * (ce1 + ce2), c * (dI_q + dI_k), c * (dT_q + dT_k), c * (ds1 + ds2)


def disco_rank(I, T, s: float, rank: int, N: int):
    """What rank `rank` of N computes in DisCo (Sec. 4.1 Eq. 4-6, Alg. 1).

    Only the two b x B logit blocks  s I_r T^T  and  s T_r I^T  are formed.
    Outputs, all carrying c = 1/(2B):
      loss_r : c * sum_{i in R_r} (ce1_i + ce2_i)
      gI_r   : B x d.  Rows R_r get the query-side term of the image->text block;
               every row gets the key-side term of the text->image block.
      gT_r   : B x d, the mirror image.
      gs_r   : this rank's share of dL/ds.
    Rows of gI_r, gT_r outside R_r are what Eq. 5/7 sends to the other ranks.
    """
    I, T = _f64(I), _f64(T)
    B = I.shape[0]
    if N <= 0 or B % N != 0 or not (0 <= rank < N):
        raise ValueError("need B % N == 0 and 0 <= rank < N")
    b = B // N
    c = 1.0 / (2.0 * B)
    R = np.arange(rank * b, (rank + 1) * b)
    ce1, dI_q, dT_k, ds1 = directional_terms(I, T, s, R)
    ce2, dT_q, dI_k, ds2 = directional_terms(T, I, s, R)
    gI = c * dI_k
    gI[R] += c * dI_q
    gT = c * dT_k
    gT[R] += c * dT_q
    return c * (ce1 + ce2), gI, gT, c * (ds1 + ds2)


def disco_all_ranks(I, T, s: float, N: int):
    """Sum of disco_rank over all ranks: what Alg. 1's all_reduce leaves behind."""
    loss, gI, gT, gs = 0.0, 0.0, 0.0, 0.0
    for r in range(N):
        l, a, t, g = disco_rank(I, T, s, r, N)
        loss, gI, gT, gs = loss + l, gI + a, gT + t, gs + g
    return loss, gI, gT, gs


def rank_row_stats(I, T, s: float, rank: int, N: int):
    """Row log-sum-exp of both logit blocks of one rank (length b each)."""
    I, T = _f64(I), _f64(T)
    b = I.shape[0] // N
    R = np.arange(rank * b, (rank + 1) * b)
    lseA = np.empty(b)
    lseC = np.empty(b)
    for lo in range(0, b, _CHUNK):
        idx = R[lo:lo + _CHUNK]
        lseA[lo:lo + idx.size] = _row_logsumexp(s * (I[idx] @ T.T))
        lseC[lo:lo + idx.size] = _row_logsumexp(s * (T[idx] @ I.T))
    return lseA, lseC


def rank_loss_from_stats(I, T, s: float, rank: int, N: int, lseA, lseC) -> float:
    """loss_r = c * sum_{i in R_r} [(lseA_i - z_ii) + (lseC_i - z_ii)],  z_ii = s <I_i, T_i>."""
    I, T = _f64(I), _f64(T)
    B = I.shape[0]
    b = B // N
    R = np.arange(rank * b, (rank + 1) * b)
    zii = s * np.sum(I[R] * T[R], axis=1)
    return float(np.sum((lseA - zii) + (lseC - zii)) / (2.0 * B))


def rank_grad_rows(I, T, s: float, rank: int, N: int, lseA, lseC, out_rows, magnitudes=False):
    """Selected rows of disco_rank's gI_r and gT_r, computed one output row at a time.

    For an output row j, gT_r[j] = c s [ sum_{i in R_r} (P^A_ij - [j=i]) I_i ]
                                  + [j in R_r] c s sum_j' (P^C_jj' - [j'=j]) I_j'
    and gI_r[j] likewise with the roles of the blocks exchanged.  Needs the row
    log-sum-exps from rank_row_stats.  Used to spot-check outputs at sizes where
    the dense disco_rank would take minutes.  With magnitudes=True every term enters by its
    absolute value, which gives the same rows of disco_rank_term_scale.
    """
    I, T = _f64(I), _f64(T)
    B, d = I.shape
    b = B // N
    c = 1.0 / (2.0 * B)
    R = np.arange(rank * b, (rank + 1) * b)
    IR, TR = I[R], T[R]
    out_rows = np.asarray(out_rows, dtype=np.int64)
    gI = np.zeros((out_rows.size, d))
    gT = np.zeros((out_rows.size, d))
    mag = (lambda a: np.abs(a)) if magnitudes else (lambda a: a)
    if magnitudes:
        s_out = abs(s)
        IR, TR, Ia, Ta = np.abs(IR), np.abs(TR), np.abs(I), np.abs(T)
    else:
        s_out, Ia, Ta = s, I, T
    IRs, TRs = I[R], T[R]                                # signed copies for the logits
    for n, j in enumerate(out_rows):
        pA = np.exp(s * (IRs @ T[j]) - lseA)             # column j of P^A, length b
        pC = np.exp(s * (TRs @ I[j]) - lseC)             # column j of P^C
        if rank * b <= j < (rank + 1) * b:
            pA[j - rank * b] -= 1.0
            pC[j - rank * b] -= 1.0
        gT[n] = c * s_out * (mag(pA) @ IR)
        gI[n] = c * s_out * (mag(pC) @ TR)
        if rank * b <= j < (rank + 1) * b:
            i = j - rank * b
            rowA = np.exp(s * (T @ I[j]) - lseA[i])      # row i of P^A over all columns
            rowA[j] -= 1.0
            rowC = np.exp(s * (I @ T[j]) - lseC[i])
            rowC[j] -= 1.0
            gI[n] += c * s_out * (mag(rowA) @ Ta)
            gT[n] += c * s_out * (mag(rowC) @ Ia)
    return gI, gT
