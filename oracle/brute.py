"""Element-by-element writing of the CLIP loss in pure Python (test infrastructure).

A second, independent writing of Eq. 1 and of the per-rank restriction
(Sec. 4.1), with explicit loops and math.exp/log only, for B <= 16.  It exists
to catch index, sign and transposition mistakes in the vectorised oracle.
"""
from __future__ import annotations

import math


def _dot(u, v):
    return math.fsum(a * b for a, b in zip(u, v))


def brute_rank(I, T, s, rank, N):
    """Loss and gradients of rank `rank` (sum convention, factor 1/(2B))."""
    B, d = len(I), len(I[0])
    b = B // N
    c = 1.0 / (2.0 * B)
    gI = [[0.0] * d for _ in range(B)]
    gT = [[0.0] * d for _ in range(B)]
    loss, gs = 0.0, 0.0
    for i in range(rank * b, (rank + 1) * b):
        # image i looks for its text among all B texts
        cos = [_dot(I[i], T[j]) for j in range(B)]
        mx = max(s * v for v in cos)
        den = math.fsum(math.exp(s * v - mx) for v in cos)
        loss += c * (mx + math.log(den) - s * cos[i])
        for j in range(B):
            g = math.exp(s * cos[j] - mx) / den - (1.0 if j == i else 0.0)
            gs += c * g * cos[j]
            for k in range(d):
                gI[i][k] += c * s * g * T[j][k]
                gT[j][k] += c * s * g * I[i][k]
        # text i looks for its image among all B images
        cos = [_dot(T[i], I[j]) for j in range(B)]
        mx = max(s * v for v in cos)
        den = math.fsum(math.exp(s * v - mx) for v in cos)
        loss += c * (mx + math.log(den) - s * cos[i])
        for j in range(B):
            g = math.exp(s * cos[j] - mx) / den - (1.0 if j == i else 0.0)
            gs += c * g * cos[j]
            for k in range(d):
                gT[i][k] += c * s * g * I[j][k]
                gI[j][k] += c * s * g * T[i][k]
    return loss, gI, gT, gs


def brute_full(I, T, s):
    return brute_rank(I, T, s, 0, 1)


def brute_rank_term_scale(I, T, s, rank, N):
    """Same loops as brute_rank with every gradient term replaced by its magnitude."""
    B, d = len(I), len(I[0])
    b = B // N
    c = 1.0 / (2.0 * B)
    aI = [[0.0] * d for _ in range(B)]
    aT = [[0.0] * d for _ in range(B)]
    for i in range(rank * b, (rank + 1) * b):
        for (Q, K, aQ, aK) in ((I, T, aI, aT), (T, I, aT, aI)):
            cos = [_dot(Q[i], K[j]) for j in range(B)]
            mx = max(s * v for v in cos)
            den = math.fsum(math.exp(s * v - mx) for v in cos)
            for j in range(B):
                g = abs(math.exp(s * cos[j] - mx) / den - (1.0 if j == i else 0.0))
                for k in range(d):
                    aQ[i][k] += c * abs(s) * g * abs(K[j][k])
                    aK[j][k] += c * abs(s) * g * abs(Q[i][k])
    return aI, aT


def brute_rank_gs_term_scale(I, T, s, rank, N):
    """Same loops as brute_rank's d/ds with every term replaced by its magnitude."""
    B = len(I)
    b = B // N
    c = 1.0 / (2.0 * B)
    total = 0.0
    for i in range(rank * b, (rank + 1) * b):
        for (Q, K) in ((I, T), (T, I)):
            cos = [_dot(Q[i], K[j]) for j in range(B)]
            mx = max(s * v for v in cos)
            den = math.fsum(math.exp(s * v - mx) for v in cos)
            for j in range(B):
                total += c * abs(math.exp(s * cos[j] - mx) / den - (1.0 if j == i else 0.0)) * abs(cos[j])
    return total


def brute_ntxent_rank(Z, s, rank, N):
    """Self-supervised (two-view) contrastive loss of rank `rank`, element by element: rows 0..M-1 and M..2M-1 are
    the two views, the positive of row i is row (i + M) mod 2M, the self-similarity is left out.  Factor 1/B."""
    B, d = len(Z), len(Z[0])
    M, b = B // 2, B // N
    g = [[0.0] * d for _ in range(B)]
    loss, gs = 0.0, 0.0
    for i in range(rank * b, (rank + 1) * b):
        p = (i + M) % B
        cos = [_dot(Z[i], Z[k]) for k in range(B)]
        others = [k for k in range(B) if k != i]
        mx = max(s * cos[k] for k in others)
        den = math.fsum(math.exp(s * cos[k] - mx) for k in others)
        loss += (mx + math.log(den) - s * cos[p]) / B
        for k in others:
            w = math.exp(s * cos[k] - mx) / den - (1.0 if k == p else 0.0)
            gs += w * cos[k] / B
            for c in range(d):
                g[i][c] += s * w * Z[k][c] / B
                g[k][c] += s * w * Z[i][c] / B
    return loss, g, gs
