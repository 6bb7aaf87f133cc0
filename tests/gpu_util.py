"""Helpers for the GPU parity tests: device buffers via torch, calls through the C ABI, tolerances."""
import numpy as np
import torch

import paper_2304_08480_amd as dl


def to_device(I_f32, T_f32, I_bits, T_bits, dtype):
    if dtype == "bf16":
        I = torch.from_numpy(I_bits.view(np.int16)).cuda()
        T = torch.from_numpy(T_bits.view(np.int16)).cuda()
        return I, T, dl.DISCO_BF16
    return torch.from_numpy(I_f32).cuda(), torch.from_numpy(T_f32).cuda(), dl.DISCO_F32


def term_scale(oc, I, T, s, rank, N):
    """(scale_gI, scale_gT, oracle_floor) for check_tensor."""
    sI, sT = oc.disco_rank_term_scale(I, T, s, rank, N)
    return sI, sT, 1e-13 * abs(s) / (2.0 * I.shape[0])


class Runner:
    """Owns outputs and workspace for one (B, d, N, dtype, path)."""

    def __init__(self, I_dev, T_dev, B, d, N, dt, path):
        self.I, self.T, self.B, self.d, self.N, self.dt, self.path = I_dev, T_dev, B, d, N, dt, path
        self.ws_bytes = dl.disco_workspace_bytes(B, d, N, dt, path)
        assert self.ws_bytes > 0, "path does not support this configuration"
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        assert self.ws.data_ptr() % 256 == 0
        self.loss = torch.full((1,), float("nan"), device="cuda")
        self.gs = torch.full((1,), float("nan"), device="cuda")
        self.gI = torch.full((B, d), float("nan"), device="cuda")
        self.gT = torch.full((B, d), float("nan"), device="cuda")

    def rank(self, r, s, accumulate=False):
        dl.disco_loss_fwd_bwd(self.I, self.T, self.B, self.d, r, self.N, s, self.dt, self.path, accumulate,
                              self.loss, self.gI, self.gT, self.gs, self.ws, self.ws_bytes,
                              torch.cuda.current_stream())

    def full(self, s):
        dl.clip_loss_fwd_bwd(self.I, self.T, self.B, self.d, s, self.dt, self.path, self.loss, self.gI, self.gT,
                             self.gs, self.ws, self.ws_bytes, torch.cuda.current_stream())

    def results(self):
        torch.cuda.synchronize()
        return (float(self.loss.item()), self.gI.cpu().numpy().astype(np.float64),
                self.gT.cpu().numpy().astype(np.float64), float(self.gs.item()))


# Tolerances.
# Scalars (loss, d/ds) and the Frobenius-relative error of each gradient tensor use the stated bars:
# 1e-4 for fp32 inputs, 2e-2 for bf16 inputs with fp32 accumulation.  (The loss never sees a bf16
# rounding, its row sums are fp32, so it keeps 1e-4 in both; d/ds gets ten times the loss bar.)
# Elementwise, TWO bounds are asserted and every entry must meet the smaller one:
#  (stated)  |error| <= abs * max|ref| + rel * |ref|, the stated bar with its absolute part taken relative to
#            the tensor's largest magnitude (a literal 1e-3 would exceed every gradient entry, which are of size
#            1/(2B) and below): rel 2e-2, abs 1e-3 for bf16; rel 1e-4, abs 1e-5 for fp32 (sequential fp32
#            accumulation of B terms alone gives about sqrt(B) * 2^-24 = 1e-6 of the largest entries);
#  (derived) every gradient entry is a sum of products, and on the bf16 path each factor of each product is
#            rounded to bf16 once (8 significant bits, unit roundoff u = 2^-8), so
#                |error_ik| <= 2u * sum_j |term_ijk|  (1 + o(1))
#            whatever cancels in the sum.  The sum of term magnitudes comes from the oracle
#            (disco_rank_term_scale); k = 2u with 10% slack = 8.6e-3.  On the fp32 path the same sum bounds the
#            accumulation error: k = 1e-5 (about 2^-24 * sqrt(terms) with slack) next to 1e-4 * |ref|.
TOL = {
    "f32": dict(scalar=1e-4, frob=1e-4, rel=1e-4, k_scale=1e-5, stated_abs=1e-5, stated_rel=1e-4),
    "bf16": dict(scalar=1e-4, frob=2e-2, rel=0.0, k_scale=8.6e-3, stated_abs=1e-3, stated_rel=2e-2),
}


def check_scalar(name, got, ref, tol, abs_tol=1e-12):
    """|got - ref| <= tol * |ref| + abs_tol.  abs_tol covers the oracle's own float64 cancellation when the
    softmax saturates (s = 100: lse - z_label is a difference of numbers near 100, good to ~1e-14 per row)."""
    err = abs(got - ref)
    assert np.isfinite(got) and err <= tol * abs(ref) + abs_tol, \
        f"{name}: got {got!r} ref {ref!r} abs err {err:.3e} > {tol} * |ref| + {abs_tol}"
    return err / max(abs(ref), abs_tol)


def check_tensor(name, got, ref, kind, scale, oracle_floor=0.0, k_extra=0.0, cancelling=False):
    """Frobenius-relative error against the stated bar, and the smaller of the two elementwise bounds.

    oracle_floor: absolute per-entry uncertainty of the float64 oracle itself.  It forms P_label - 1 by
    subtraction, so when the softmax saturates (P_label = 1 - 1e-29 at s = 100) its gradient entries are
    rounding noise of size 2^-53 * c * s rather than the true 1e-30; callers pass 1e-13 * c * s.
    k_extra: added to the factor of the derived bound.  A logit held in fp32 is good to |z| * 2^-24, which moves
    every softmax term by that relative amount; tests whose logits are far larger than CLIP's (features of norm
    above 1) pass 2^-22 * max|z|.  Zero for every CLIP-like input.
    cancelling: the inputs are built so that the terms of a gradient entry cancel (a duplicate pair ties with the
    positive, so that (P_ii - 1) y_i + P_ij y_j is a small residual of two terms of size 1/2; entries 25 times
    smaller than the sum of their term magnitudes next to entries with none).  The stated relative bars presume
    gradients that are not small residuals of large terms: rounding P to bf16, which the bf16 arithmetic
    prescribes, then costs more than 2e-2 of the residual.  With cancelling=True the absolute part of the stated
    elementwise bound is the literal one (not relative to the largest entry) and the Frobenius error may also be
    within the derived bound's norm, k * |scale|_F; the derived elementwise bound is asserted unchanged.
    """
    t = TOL[kind]
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    diff = np.abs(got - ref)
    nd, nr = np.linalg.norm(got - ref), np.linalg.norm(ref)
    fro = nd / max(nr, 1e-300)
    frob_limit = t["frob"] * nr
    if cancelling:
        frob_limit = max(frob_limit, (t["k_scale"] + k_extra) * np.linalg.norm(scale))
    assert nd <= frob_limit + oracle_floor * np.sqrt(ref.size), f"{name}: Frobenius rel err {fro:.3e} > {t['frob']}"
    derived = t["rel"] * np.abs(ref) + (t["k_scale"] + k_extra) * scale
    stated = t["stated_abs"] * (1.0 if cancelling else np.abs(ref).max()) + t["stated_rel"] * np.abs(ref)
    bound = np.minimum(derived, stated) + oracle_floor + 1e-300
    ratio = (diff / bound).max()
    w = np.unravel_index(np.argmax(diff / bound), diff.shape)
    assert ratio <= 1.0, (f"{name}: elementwise error reaches {ratio:.2f} x its bound at {w}: diff {diff[w]:.3e}, ref {ref[w]:.3e}, "
                          f"derived bound {derived[w]:.3e}, stated bound {stated[w]:.3e}, max|ref| {np.abs(ref).max():.3e}; "
                          f"largest diff/derived {(diff / (derived + oracle_floor + 1e-300)).max():.2f}, "
                          f"largest diff/stated {(diff / (stated + oracle_floor + 1e-300)).max():.2f}")
    return fro, ratio
