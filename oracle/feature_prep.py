"""Plain float64 NumPy oracle of the two steps on either side of the loss (test infrastructure only).

In the paper's Alg. 1 the encoders hand features to the loss and receive the feature gradients back
(first segment "I_n, T_n = ...", last segment "backward on features"); the text neither prints the
row normalisation of those features nor the parametrisation of the logit multiplier `t`.  Reading
taken (CLIP's convention, which the paper builds on, Sec. 5.1):

  * features are L2-normalised row by row:  u = x / max(|x|, eps), eps = 1e-12;
  * the multiplier is s = min(exp(theta), s_max) with a learnable theta and the cap s_max = 100.

Backward of the normalisation for an upstream gradient g (d loss / d u):
    |x| > eps :  d loss / d x = (g - <g, u> u) / |x|        (Jacobian (I - u u^T) / |x|)
    otherwise :  d loss / d x = g / eps                       (the cap is active: u = x / eps)
Backward of the multiplier:  d s / d theta = exp(theta) where exp(theta) <= s_max, else 0.

Each function is the definition written out; tests/test_oracle_prep_pins.py pins them to closed forms,
finite differences, orthogonality/scaling identities and a library autograd routine.
"""
from __future__ import annotations

import math

import numpy as np

EPS = 1e-12


def l2_normalize_fwd(X):
    """u_i = x_i / max(|x_i|, eps) for every row.  Returns (U, inv) with inv_i = 1 / max(|x_i|, eps)."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    n = np.sqrt((X * X).sum(axis=1))
    inv = 1.0 / np.maximum(n, EPS)
    return X * inv[:, None], inv


def l2_normalize_bwd(G, X):
    """d loss / d x for rows x with upstream gradient G = d loss / d u (same shape)."""
    G = np.ascontiguousarray(G, dtype=np.float64)
    X = np.ascontiguousarray(X, dtype=np.float64)
    n = np.sqrt((X * X).sum(axis=1))
    out = np.empty_like(X)
    live = n > EPS
    u = X[live] / n[live, None]
    g = G[live]
    out[live] = (g - (g * u).sum(axis=1)[:, None] * u) / n[live, None]
    out[~live] = G[~live] / EPS
    return out


def logit_scale_fwd(theta: float, s_max: float = 100.0) -> float:
    """s = min(exp(theta), s_max)."""
    return min(math.exp(theta), s_max)


def logit_scale_bwd(theta: float, gs: float, s_max: float = 100.0) -> float:
    """d loss / d theta given gs = d loss / d s."""
    e = math.exp(theta)
    return gs * e if e <= s_max else 0.0
