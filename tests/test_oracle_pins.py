"""Pins of the float64 oracle against things other than itself.

Each test names the passage or the mathematics that fixes the expected value.
None of these needs a GPU.
"""
import math

import numpy as np
import pytest
import torch

from oracle import brute, clip_oracle as oc
from synth import clip_pairs


def _rand_pairs(B, d, seed):
    I, T = clip_pairs(B, d, seed)
    return I.astype(np.float64), T.astype(np.float64)


# ---------------------------------------------------------------- closed forms
def test_all_equal_features_gives_log_B():
    # every logit equals s, so each row softmax is uniform: L = log B, no gradient
    B, d, s = 24, 7, 9.5
    u = np.zeros(d); u[2] = 1.0
    I = np.tile(u, (B, 1)); T = I.copy()
    L, gI, gT, gs = oc.clip_loss_full(I, T, s)
    assert L == pytest.approx(math.log(B), rel=1e-14)
    # d/dI_i = (s/2B) [sum_j P_ij T_j - T_i + ...] = 0 because all T_j are the same vector
    assert np.abs(gI).max() < 1e-15 and np.abs(gT).max() < 1e-15
    assert abs(gs) < 1e-15


def test_orthonormal_basis_closed_form():
    # I = T = first B basis vectors: S = identity.  Row softmax has p on the diagonal, q elsewhere.
    B, d, s = 6, 9, 3.25
    I = np.eye(B, d); T = np.eye(B, d)
    Z = math.exp(s) + B - 1
    p, q = math.exp(s) / Z, 1.0 / Z
    L, gI, gT, gs = oc.clip_loss_full(I, T, s)
    assert L == pytest.approx(math.log(Z) - s, rel=1e-14)
    assert gs == pytest.approx(-(B - 1) / Z, rel=1e-13)
    expect = np.zeros((B, d))
    for i in range(B):
        expect[i, :B] = (s / B) * q
        expect[i, i] = (s / B) * (p - 1.0)
    np.testing.assert_allclose(gI, expect, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(gT, expect, rtol=1e-13, atol=1e-16)
    # every rank holds the same share of the loss
    for N in (1, 2, 3, 6):
        for r in range(N):
            assert oc.disco_rank(I, T, s, r, N)[0] == pytest.approx(L / N, rel=1e-13)


def test_zero_scale_closed_form():
    # s = 0: uniform softmax, L = log B, no feature gradient, gs = (1/B)[(1/B) sum_ij S_ij - tr S]
    I, T = _rand_pairs(10, 5, 3)
    B = 10
    L, gI, gT, gs = oc.clip_loss_full(I, T, 0.0)
    S = I @ T.T
    assert L == pytest.approx(math.log(B), rel=1e-14)
    assert np.abs(gI).max() == 0 and np.abs(gT).max() == 0
    assert gs == pytest.approx((S.sum() / B - np.trace(S)) / B, rel=1e-12)


def test_two_pairs_by_hand():
    # B=2, d=1: logits are +-s products; written out with scalar math
    I = np.array([[1.0], [-0.5]]); T = np.array([[0.8], [0.3]]); s = 2.0
    S = [[0.8, 0.3], [-0.4, -0.15]]
    def ce(row, k):
        return math.log(sum(math.exp(s * v) for v in row)) - s * row[k]
    expect = (ce(S[0], 0) + ce(S[1], 1) + ce([S[0][0], S[1][0]], 0) + ce([S[0][1], S[1][1]], 1)) / 4.0
    assert oc.clip_loss_full(I, T, s)[0] == pytest.approx(expect, rel=1e-14)


# ------------------------------------------------------ library special cases
def test_row_logsumexp_matches_scipy():
    from scipy.special import logsumexp
    rng = np.random.default_rng(0)
    Z = rng.standard_normal((13, 37)) * 40.0
    np.testing.assert_allclose(oc._row_logsumexp(Z), logsumexp(Z, axis=1), rtol=1e-14)


def _alg1_autograd(I, T, s, rank, N):
    """The paper's Alg. 1 for one rank, transcribed with a library autograd (float64).

    logits_i = dot(I_E[rank], T_E) * t ; labels = arange(b) + b*rank ;
    loss = (CE(logits_i) + CE(logits_t)) / 2 ; loss.backward().
    Returns Alg. 1's own normalisation (mean over the rank's b rows).
    """
    It = torch.tensor(I, dtype=torch.float64, requires_grad=True)
    Tt = torch.tensor(T, dtype=torch.float64, requires_grad=True)
    st = torch.tensor(s, dtype=torch.float64, requires_grad=True)
    b = I.shape[0] // N
    sl = slice(rank * b, (rank + 1) * b)
    logits_i = (It[sl] @ Tt.T) * st
    logits_t = (Tt[sl] @ It.T) * st
    labels = torch.arange(b) + b * rank
    ce = torch.nn.functional.cross_entropy
    loss = (ce(logits_i, labels) + ce(logits_t, labels)) / 2
    loss.backward()
    return loss.item(), It.grad.numpy(), Tt.grad.numpy(), st.grad.item()


@pytest.mark.parametrize("B,d,N,s", [(12, 5, 3, 4.0), (16, 8, 4, 14.285714), (8, 4, 1, 100.0), (9, 3, 9, 1.0)])
def test_rank_matches_alg1_autograd(B, d, N, s):
    # Alg. 1 averages over b rows and later over N ranks (all_reduce AVG): per-rank value / N = sum convention
    I, T = _rand_pairs(B, d, B + N)
    for r in range(N):
        L, gI, gT, gs = _alg1_autograd(I, T, s, r, N)
        l, a, t, g = oc.disco_rank(I, T, s, r, N)
        assert l == pytest.approx(L / N, rel=1e-12)
        # atol: at s = 100 entries of size 1e-7 come from cancelling O(1) terms
        np.testing.assert_allclose(a, gI / N, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(t, gT / N, rtol=1e-10, atol=1e-13)
        assert g == pytest.approx(gs / N, rel=1e-10, abs=1e-16)


def test_full_matches_autograd_of_original_clip():
    # Eq. 1 / Fig. 1: the whole B x B matrix on one device
    I, T = _rand_pairs(20, 6, 5)
    L, gI, gT, gs = _alg1_autograd(I, T, 7.0, 0, 1)
    l, a, t, g = oc.clip_loss_full(I, T, 7.0)
    assert l == pytest.approx(L, rel=1e-13)
    np.testing.assert_allclose(a, gI, rtol=1e-10, atol=1e-16)
    np.testing.assert_allclose(t, gT, rtol=1e-10, atol=1e-16)
    assert g == pytest.approx(gs, rel=1e-10)


# ------------------------------------------------------------------ brute force
@pytest.mark.parametrize("B,d,N", [(8, 4, 2), (6, 3, 3), (4, 5, 1)])
def test_vectorised_matches_pure_loops(B, d, N):
    I, T = _rand_pairs(B, d, 11)
    s = 5.5
    for r in range(N):
        bl, bI, bT, bs = brute.brute_rank(I.tolist(), T.tolist(), s, r, N)
        l, a, t, g = oc.disco_rank(I, T, s, r, N)
        assert l == pytest.approx(bl, rel=1e-12)
        np.testing.assert_allclose(a, np.array(bI), rtol=1e-11, atol=1e-15)
        np.testing.assert_allclose(t, np.array(bT), rtol=1e-11, atol=1e-15)
        assert g == pytest.approx(bs, rel=1e-11)
    bl, bI, bT, bs = brute.brute_full(I.tolist(), T.tolist(), s)
    l, a, t, g = oc.clip_loss_full(I, T, s)
    assert l == pytest.approx(bl, rel=1e-12)
    np.testing.assert_allclose(a, np.array(bI), rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(t, np.array(bT), rtol=1e-11, atol=1e-15)
    assert g == pytest.approx(bs, rel=1e-11)


# ---------------------------------------------------------- finite differences
@pytest.mark.parametrize("B,d,N", [(8, 4, 2), (12, 5, 3)])
def test_gradients_by_central_differences(B, d, N):
    # perturb raw entries (no re-normalisation) of the loss value; every entry of gI, gT and gs
    I, T = _rand_pairs(B, d, 21)
    s, h = 6.0, 1e-6
    for r in range(N):
        f = lambda I_, T_, s_: oc.disco_rank(I_, T_, s_, r, N)[0]
        _, gI, gT, gs = oc.disco_rank(I, T, s, r, N)
        for (arr, grad, which) in ((I, gI, 0), (T, gT, 1)):
            fd = np.zeros_like(arr)
            for i in range(B):
                for k in range(d):
                    p, m = arr.copy(), arr.copy()
                    p[i, k] += h; m[i, k] -= h
                    args_p = (p, T, s) if which == 0 else (I, p, s)
                    args_m = (m, T, s) if which == 0 else (I, m, s)
                    fd[i, k] = (f(*args_p) - f(*args_m)) / (2 * h)
            np.testing.assert_allclose(grad, fd, rtol=2e-7, atol=2e-10)
        fd_s = (f(I, T, s + h) - f(I, T, s - h)) / (2 * h)
        assert gs == pytest.approx(fd_s, rel=1e-7, abs=1e-10)


# ------------------------------------------------- the paper's own invariants
@pytest.mark.parametrize("N", [1, 2, 4, 16])
def test_rank_sum_equals_full_loss(N):
    # Eq. 3: L_d equals L; Eq. 4-7: intra + collected inter gradients equal the full gradient
    I, T = _rand_pairs(16, 6, 2)
    s = 12.0
    L, gI, gT, gs = oc.clip_loss_full(I, T, s)
    l, a, t, g = oc.disco_all_ranks(I, T, s, N)
    assert l == pytest.approx(L, rel=1e-13)
    np.testing.assert_allclose(a, gI, rtol=1e-11, atol=1e-17)
    np.testing.assert_allclose(t, gT, rtol=1e-11, atol=1e-17)
    assert g == pytest.approx(gs, rel=1e-12)


def test_foreign_rows_come_only_from_the_other_direction():
    # Sec. 4.1: L1(I_nbar, T_A) induces no gradient on I_n.  So in rank r's gI, the rows outside R_r are
    # exactly the key-side term of the text->image block, and they are not zero in general.
    I, T = _rand_pairs(12, 5, 9)
    s, N, r = 8.0, 3, 1
    b = 4
    R = np.arange(r * b, (r + 1) * b)
    out = np.setdiff1d(np.arange(12), R)
    _, gI, gT, _ = oc.disco_rank(I, T, s, r, N)
    c = 1 / 24
    _, _, dI_k, _ = oc.directional_terms(T, I, s, R)     # text->image block, key side = images
    _, _, dT_k, _ = oc.directional_terms(I, T, s, R)
    np.testing.assert_allclose(gI[out], c * dI_k[out], rtol=1e-13)
    np.testing.assert_allclose(gT[out], c * dT_k[out], rtol=1e-13)
    assert np.abs(gI[out]).min() > 0 and np.abs(gT[out]).min() > 0


def test_homogeneity_identity():
    # the loss depends on (I, T, s) only through s * I T^T, so <gI, I> = <gT, T> = s * gs (per rank too)
    I, T = _rand_pairs(16, 7, 4)
    s = 9.0
    for N in (1, 4):
        for r in range(N):
            _, gI, gT, gs = oc.disco_rank(I, T, s, r, N)
            assert np.sum(gI * I) == pytest.approx(s * gs, rel=1e-11)
            assert np.sum(gT * T) == pytest.approx(s * gs, rel=1e-11)


def test_rotation_and_swap_symmetries():
    I, T = _rand_pairs(10, 6, 6)
    s = 5.0
    L, gI, gT, gs = oc.clip_loss_full(I, T, s)
    Q, _ = np.linalg.qr(np.random.default_rng(1).standard_normal((6, 6)))
    L2, gI2, gT2, gs2 = oc.clip_loss_full(I @ Q, T @ Q, s)
    assert L2 == pytest.approx(L, rel=1e-13) and gs2 == pytest.approx(gs, rel=1e-11)
    np.testing.assert_allclose(gI2, gI @ Q, rtol=1e-9, atol=1e-15)
    # exchanging the roles of images and texts exchanges the gradients
    L3, gI3, gT3, gs3 = oc.clip_loss_full(T, I, s)
    assert L3 == pytest.approx(L, rel=1e-13) and gs3 == pytest.approx(gs, rel=1e-12)
    np.testing.assert_allclose(gI3, gT, rtol=1e-11, atol=1e-17)
    np.testing.assert_allclose(gT3, gI, rtol=1e-11, atol=1e-17)


def test_large_scale_is_finite_and_positive():
    # s = 100 (the clamp of CLIP's multiplier): exp overflows without max subtraction
    I, T = _rand_pairs(32, 8, 8)
    L, gI, gT, gs = oc.clip_loss_full(I, T, 100.0)
    assert np.isfinite(L) and L >= 0 and np.isfinite(gI).all() and np.isfinite(gs)


def test_sampled_rows_match_dense():
    I, T = _rand_pairs(24, 6, 13)
    s, N, r = 7.0, 3, 2
    _, gI, gT, _ = oc.disco_rank(I, T, s, r, N)
    lseA, lseC = oc.rank_row_stats(I, T, s, r, N)
    rows = np.array([0, 5, 16, 19, 23])
    a, t = oc.rank_grad_rows(I, T, s, r, N, lseA, lseC, rows)
    np.testing.assert_allclose(a, gI[rows], rtol=1e-11, atol=1e-17)
    np.testing.assert_allclose(t, gT[rows], rtol=1e-11, atol=1e-17)
    assert oc.rank_loss_from_stats(I, T, s, r, N, lseA, lseC) == pytest.approx(oc.disco_rank(I, T, s, r, N)[0], rel=1e-13)


def test_memory_model_figures_from_the_paper():
    # tests/golden/memory_model.txt holds the figures printed in Sec. 1, 3 and 4.1
    import os
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "memory_model.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()[:2]
                vals[k] = float(v)
    B = 65536
    assert B * B == pytest.approx(vals["sim_entries_B65536"], rel=0.01)
    assert B * B * 4 / 2**30 == vals["sim_gib_f32_B65536"]
    for N, key in ((16, "saved_fraction_N16"), (64, "saved_fraction_N64")):
        full, disco = B * B, 2 * (B // N) * B
        assert 1 - disco / full == vals[key]
    assert round(100 * vals["saved_fraction_N64"]) == vals["saved_percent_N64_approx"]


def test_term_scale_matches_loops_and_bounds_the_gradient():
    I, T = _rand_pairs(8, 4, 17)
    s, N = 6.5, 2
    for r in range(N):
        sI, sT = oc.disco_rank_term_scale(I, T, s, r, N)
        bI, bT = brute.brute_rank_term_scale(I.tolist(), T.tolist(), s, r, N)
        np.testing.assert_allclose(sI, np.array(bI), rtol=1e-11)
        np.testing.assert_allclose(sT, np.array(bT), rtol=1e-11)
        _, gI, gT, _ = oc.disco_rank(I, T, s, r, N)
        assert (np.abs(gI) <= sI * (1 + 1e-12)).all() and (np.abs(gT) <= sT * (1 + 1e-12)).all()   # triangle inequality
    # sampled rows agree with the dense arrays
    lseA, lseC = oc.rank_row_stats(I, T, s, 1, N)
    rows = np.array([0, 3, 4, 7])
    a, t = oc.rank_grad_rows(I, T, s, 1, N, lseA, lseC, rows, magnitudes=True)
    sI, sT = oc.disco_rank_term_scale(I, T, s, 1, N)
    np.testing.assert_allclose(a, sI[rows], rtol=1e-11)
    np.testing.assert_allclose(t, sT[rows], rtol=1e-11)


def test_gs_term_scale_matches_loops_and_bounds_gs():
    I, T = _rand_pairs(8, 4, 23)
    s, N = 4.5, 2
    for r in range(N):
        sc = oc.disco_rank_gs_term_scale(I, T, s, r, N)
        assert sc == pytest.approx(brute.brute_rank_gs_term_scale(I.tolist(), T.tolist(), s, r, N), rel=1e-11)
        assert abs(oc.disco_rank(I, T, s, r, N)[3]) <= sc * (1 + 1e-12)          # triangle inequality
    # s = 0: P = 1/B everywhere, so the scale is c * sum_ij |1/B - [j = i]| |S_ij| over both directions
    B = I.shape[0]
    S = I.astype(np.float64) @ T.astype(np.float64).T
    W = np.abs(1.0 / B - np.eye(B))
    want = (np.sum(W * np.abs(S)) + np.sum(W * np.abs(S.T))) / (2.0 * B)
    assert oc.disco_rank_gs_term_scale(I, T, 0.0, 0, 1) == pytest.approx(want, rel=1e-12)
