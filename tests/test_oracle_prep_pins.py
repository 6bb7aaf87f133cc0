"""Pins of the feature-preparation oracle (row L2 normalisation, logit-multiplier parametrisation) against
closed forms, finite differences, identities and a library routine.  No GPU needed."""
import math

import numpy as np
import pytest
import torch

from oracle import clip_oracle as oc
from oracle import feature_prep as fp


def _rng(seed):
    return np.random.default_rng(seed)


def test_forward_closed_form_3_4_5():
    U, inv = fp.l2_normalize_fwd(np.array([[3.0, 4.0], [0.0, -2.0], [1e-3, 0.0]]))
    assert np.allclose(U, [[0.6, 0.8], [0.0, -1.0], [1.0, 0.0]], rtol=1e-15, atol=0)
    assert np.allclose(inv, [0.2, 0.5, 1e3], rtol=1e-15)


def test_forward_rows_are_unit_and_parallel():
    X = _rng(0).normal(size=(17, 9)) * 3.7
    U, inv = fp.l2_normalize_fwd(X)
    assert np.allclose((U * U).sum(axis=1), 1.0, rtol=1e-14)
    # parallel to the input with a positive factor
    assert np.allclose(U * np.sqrt((X * X).sum(axis=1))[:, None], X, rtol=1e-13)
    assert np.all(inv > 0)


def test_zero_row_uses_the_cap():
    X = np.zeros((2, 4)); X[1] = [2.0, 0, 0, 0]
    U, inv = fp.l2_normalize_fwd(X)
    assert np.all(U[0] == 0) and inv[0] == 1.0 / fp.EPS
    G = np.array([[1.0, -2.0, 0.5, 0.0], [1.0, 1.0, 1.0, 1.0]])
    D = fp.l2_normalize_bwd(G, X)
    assert np.allclose(D[0], G[0] / fp.EPS)
    assert np.allclose(D[1], [0.0, 0.5, 0.5, 0.5])          # (g - g_0 e_0) / 2


def test_backward_matches_central_differences():
    rng = _rng(1)
    X = rng.normal(size=(5, 6)); G = rng.normal(size=(5, 6))
    D = fp.l2_normalize_bwd(G, X)
    h = 1e-6
    for i in range(5):
        for k in range(6):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, k] += h; Xm[i, k] -= h
            fd = ((G * fp.l2_normalize_fwd(Xp)[0]).sum() - (G * fp.l2_normalize_fwd(Xm)[0]).sum()) / (2 * h)
            assert D[i, k] == pytest.approx(fd, rel=1e-7, abs=1e-9)


def test_backward_is_orthogonal_to_x_and_scales_inversely():
    rng = _rng(2)
    X = rng.normal(size=(8, 11)); G = rng.normal(size=(8, 11))
    D = fp.l2_normalize_bwd(G, X)
    assert np.abs((D * X).sum(axis=1)).max() < 1e-14          # u(x) is scale invariant: no radial component
    assert np.allclose(fp.l2_normalize_bwd(G, 2.5 * X), D / 2.5, rtol=1e-13)
    # a gradient along u itself is annihilated
    U, _ = fp.l2_normalize_fwd(X)
    assert np.abs(fp.l2_normalize_bwd(U, X)).max() < 1e-15


def test_against_library_autograd():
    rng = _rng(3)
    X = rng.normal(size=(6, 7)); G = rng.normal(size=(6, 7))
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    U = torch.nn.functional.normalize(Xt, dim=1, eps=fp.EPS)
    (U * torch.tensor(G)).sum().backward()
    assert np.allclose(fp.l2_normalize_fwd(X)[0], U.detach().numpy(), rtol=1e-14)
    assert np.allclose(fp.l2_normalize_bwd(G, X), Xt.grad.numpy(), rtol=1e-12, atol=1e-15)


def test_logit_scale_values_and_cap():
    assert fp.logit_scale_fwd(math.log(1 / 0.07)) == pytest.approx(1 / 0.07, rel=1e-15)
    assert fp.logit_scale_fwd(5.0) == 100.0                    # exp(5) = 148.4 is capped
    assert fp.logit_scale_bwd(5.0, 3.0) == 0.0
    th = 1.3
    h = 1e-6
    fd = (fp.logit_scale_fwd(th + h) - fp.logit_scale_fwd(th - h)) / (2 * h)
    assert fp.logit_scale_bwd(th, 2.0) == pytest.approx(2.0 * fd, rel=1e-9)
    assert fp.logit_scale_bwd(math.log(100.0) - 1e-9, 1.0) == pytest.approx(100.0, rel=1e-8)


def test_chain_through_the_loss_matches_central_differences():
    # L(theta, Xi, Xt) = clip loss of the normalised features at s = min(exp theta, 100)
    rng = _rng(4)
    B, d, theta = 6, 5, 1.1
    Xi = rng.normal(size=(B, d)); Xt = Xi + 0.5 * rng.normal(size=(B, d))

    def loss(Xi_, Xt_, th):
        return oc.clip_loss_full(fp.l2_normalize_fwd(Xi_)[0], fp.l2_normalize_fwd(Xt_)[0], fp.logit_scale_fwd(th))[0]

    I, T = fp.l2_normalize_fwd(Xi)[0], fp.l2_normalize_fwd(Xt)[0]
    _, gI, gT, gs = oc.clip_loss_full(I, T, fp.logit_scale_fwd(theta))
    dXi, dXt = fp.l2_normalize_bwd(gI, Xi), fp.l2_normalize_bwd(gT, Xt)
    dth = fp.logit_scale_bwd(theta, gs)
    h = 1e-6
    assert dth == pytest.approx((loss(Xi, Xt, theta + h) - loss(Xi, Xt, theta - h)) / (2 * h), rel=1e-7)
    for (i, k) in [(0, 0), (2, 3), (5, 4)]:
        P, M = Xi.copy(), Xi.copy(); P[i, k] += h; M[i, k] -= h
        assert dXi[i, k] == pytest.approx((loss(P, Xt, theta) - loss(M, Xt, theta)) / (2 * h), rel=1e-6, abs=1e-10)
        P, M = Xt.copy(), Xt.copy(); P[i, k] += h; M[i, k] -= h
        assert dXt[i, k] == pytest.approx((loss(Xi, P, theta) - loss(Xi, M, theta)) / (2 * h), rel=1e-6, abs=1e-10)
