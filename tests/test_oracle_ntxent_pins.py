"""Pins of the self-supervised (two-view) contrastive-loss oracle: closed forms, brute-force loops, central finite
differences of every gradient entry, a library autograd transcription, and the decomposition's rank-sum equality
(Sec. 4.1: the per-rank results summed over the ranks are the non-decomposed loss and gradients)."""
import math

import numpy as np
import pytest
import torch

from oracle import brute
from oracle import ntxent_oracle as nx


def _views(M, d, seed, noise=0.4):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((M, d))
    b = a + noise * rng.standard_normal((M, d))
    Z = np.concatenate([a, b])
    return Z / np.linalg.norm(Z, axis=1, keepdims=True)


def test_all_rows_equal_gives_log_of_the_number_of_negatives_plus_one():
    B, d, s = 12, 5, 7.0
    u = np.zeros(d); u[2] = 1.0
    Z = np.tile(u, (B, 1))
    L, g, gs = nx.ntxent_full(Z, s)
    assert L == pytest.approx(math.log(B - 1), rel=1e-14)          # B - 1 equal logits, one of them the positive
    # every row's gradient is s/B * (mean of the other rows - positive) plus the mirror term: all rows equal -> 0
    assert np.abs(g).max() < 1e-15 and abs(gs) < 1e-15


def test_two_rows_have_no_negatives():
    Z = _views(1, 6, 3)
    L, g, gs = nx.ntxent_full(Z, 9.0)
    assert abs(L) < 1e-15 and np.abs(g).max() < 1e-15 and abs(gs) < 1e-15


def test_identical_orthonormal_views_closed_form():
    # z_i = z_{i+M} = e_i: the positive logit is s, the other B - 2 logits are 0
    M, d, s = 4, 6, 3.0
    B = 2 * M
    Z = np.zeros((B, d))
    for i in range(M):
        Z[i, i] = Z[i + M, i] = 1.0
    L, g, gs = nx.ntxent_full(Z, s)
    den = math.exp(s) + B - 2
    assert L == pytest.approx(math.log(den) - s, rel=1e-14)
    assert gs == pytest.approx(math.exp(s) / den - 1.0, rel=1e-13)   # only the positive has a non-zero cosine: (P_pos - 1) * 1
    # row i: query side (s/B)[(p - 1) e_i + q sum_{k != i, p(i)} z_k], key side the same by symmetry of this input
    p, q = math.exp(s) / den, 1.0 / den
    want = np.zeros((B, d))
    for i in range(B):
        for k in range(B):
            if k == i:
                continue
            w = (p - 1.0) if k == (i + M) % B else q
            want[i] += s / B * w * Z[k]
            want[k] += s / B * w * Z[i]
    np.testing.assert_allclose(g, want, rtol=1e-13, atol=1e-16)


@pytest.mark.parametrize("M,d,N,s", [(3, 4, 1, 5.0), (4, 3, 2, 2.5), (4, 5, 8, 11.0), (6, 4, 3, 0.0)])
def test_matches_brute_force_loops(M, d, N, s):
    Z = _views(M, d, 5 + M)
    for r in range(N):
        L, g, gs = nx.ntxent_rank(Z, s, r, N)
        bl, bg, bs = brute.brute_ntxent_rank(Z.tolist(), s, r, N)
        assert L == pytest.approx(bl, rel=1e-12, abs=1e-15) and gs == pytest.approx(bs, rel=1e-11, abs=1e-15)
        np.testing.assert_allclose(g, np.array(bg), rtol=1e-11, atol=1e-15)


def test_central_differences_of_every_entry():
    M, d, N, s, h = 4, 3, 2, 3.5, 1e-6
    Z = _views(M, d, 11)
    for r in range(N):
        L, g, gs = nx.ntxent_rank(Z, s, r, N)
        num = np.zeros_like(Z)
        for i in range(Z.shape[0]):
            for c in range(d):
                Zp, Zm = Z.copy(), Z.copy()
                Zp[i, c] += h; Zm[i, c] -= h
                num[i, c] = (nx.ntxent_rank(Zp, s, r, N)[0] - nx.ntxent_rank(Zm, s, r, N)[0]) / (2 * h)
        np.testing.assert_allclose(g, num, rtol=2e-7, atol=1e-9)
        num_s = (nx.ntxent_rank(Z, s + h, r, N)[0] - nx.ntxent_rank(Z, s - h, r, N)[0]) / (2 * h)
        assert gs == pytest.approx(num_s, rel=1e-7, abs=1e-10)


def test_library_autograd_of_masked_cross_entropy():
    # the textbook statement: cross-entropy of the logits with the diagonal masked, targets (i + M) mod B, mean over rows
    M, d, s = 5, 4, 6.0
    Z = _views(M, d, 21)
    B = 2 * M
    z = torch.tensor(Z, dtype=torch.float64, requires_grad=True)
    sc = torch.tensor(s, dtype=torch.float64, requires_grad=True)
    logits = sc * (z @ z.T)
    logits = logits.masked_fill(torch.eye(B, dtype=torch.bool), float("-inf"))
    target = (torch.arange(B) + M) % B
    loss = torch.nn.functional.cross_entropy(logits, target)
    loss.backward()
    L, g, gs = nx.ntxent_full(Z, s)
    assert L == pytest.approx(loss.item(), rel=1e-13)
    np.testing.assert_allclose(g, z.grad.numpy(), rtol=1e-11, atol=1e-15)
    assert gs == pytest.approx(sc.grad.item(), rel=1e-11)


@pytest.mark.parametrize("N", [1, 2, 4, 12])
def test_rank_sum_equals_the_full_loss(N):
    M, d, s = 6, 5, 8.0
    Z = _views(M, d, 31)
    L, g, gs = nx.ntxent_full(Z, s)
    parts = [nx.ntxent_rank(Z, s, r, N) for r in range(N)]
    assert sum(p[0] for p in parts) == pytest.approx(L, rel=1e-13)
    np.testing.assert_allclose(sum(p[1] for p in parts), g, rtol=1e-12, atol=1e-16)
    assert sum(p[2] for p in parts) == pytest.approx(gs, rel=1e-12)
    # homogeneity of the loss in (Z, s): <gZ_r, Z> = 2 s gs_r for every rank (Z enters every logit twice)
    for (l, gr, gsr) in parts:
        assert float(np.sum(gr * Z)) == pytest.approx(2.0 * s * gsr, rel=1e-11, abs=1e-14)


def test_term_scale_bounds_the_gradient_and_matches_loops():
    M, d, N, s = 4, 3, 2, 4.0
    Z = _views(M, d, 41)
    for r in range(N):
        a, aS = nx.ntxent_rank_term_scale(Z, s, r, N)
        _, g, gs = nx.ntxent_rank(Z, s, r, N)
        assert (np.abs(g) <= a * (1 + 1e-12)).all() and abs(gs) <= aS * (1 + 1e-12)
        # loops: the same sums with magnitudes
        B, b = 2 * M, 2 * M // N
        want = np.zeros_like(Z); wantS = 0.0
        for i in range(r * b, (r + 1) * b):
            cos = Z[i] @ Z.T
            oth = [k for k in range(B) if k != i]
            e = np.exp(s * cos[oth] - np.max(s * cos[oth])); P = e / e.sum()
            for w, k in zip(P, oth):
                w = abs(w - (1.0 if k == (i + M) % B else 0.0))
                want[i] += abs(s) * w * np.abs(Z[k]) / B
                want[k] += abs(s) * w * np.abs(Z[i]) / B
                wantS += w * abs(cos[k]) / B
        np.testing.assert_allclose(a, want, rtol=1e-12)
        assert aS == pytest.approx(wantS, rel=1e-12)
