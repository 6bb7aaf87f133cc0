"""GPU parity of the bf16 MFMA path on rank shares that are not whole 256-row tiles (Alg. 1 places no condition
on the local batch size): the library pads the operands to whole tiles inside its workspace, leaves the padding
out of every softmax and sum, and writes only the rows that exist.  Dense against the float64 oracle, single
ranks and the accumulated result; outputs are allocated with a guard band behind them that must stay untouched."""
import numpy as np
import pytest
import torch

import paper_2304_08480_amd as dl
from oracle import clip_oracle as oc
from synth import clip_pairs, adversarial_pairs, f32_to_bf16_bits, bf16_bits_to_f32
from tests.gpu_util import Runner, term_scale, check_scalar, check_tensor, to_device, TOL

pytestmark = pytest.mark.gpu

GUARD = -777.0


class GuardedRunner(Runner):
    """Runner whose gradient outputs are the front of larger buffers pre-filled with a sentinel."""

    def __init__(self, I_dev, T_dev, B, d, N, dt, path):
        super().__init__(I_dev, T_dev, B, d, N, dt, path)
        self._gI_all = torch.full(((B + 256) * d,), GUARD, dtype=torch.float32, device="cuda")
        self._gT_all = torch.full(((B + 256) * d,), GUARD, dtype=torch.float32, device="cuda")
        self.gI = self._gI_all[: B * d].view(B, d)
        self.gT = self._gT_all[: B * d].view(B, d)
        self.gI.zero_()
        self.gT.zero_()
        self._n = B * d

    def guards_intact(self):
        return bool((self._gI_all[self._n:] == GUARD).all().item()) and bool((self._gT_all[self._n:] == GUARD).all().item())


def _inputs(B, d, seed, kind=None, **kw):
    I, T = adversarial_pairs(B, d, seed, kind) if kind else clip_pairs(B, d, seed, **kw)
    Ib, Tb = f32_to_bf16_bits(I), f32_to_bf16_bits(T)
    return bf16_bits_to_f32(Ib), bf16_bits_to_f32(Tb), Ib, Tb


def _compare(run, ref, scale, tag, cancelling=False, gs_scale=0.0, zmax=0.0):
    eps_z = max(zmax * 2.0 ** -22, 1e-12)
    loss, gI, gT, gs = run.results()
    gs_tol, gs_abs = (TOL["bf16"]["frob"], 1e-9 + (2.0 ** -8 + eps_z) * gs_scale) if cancelling else (TOL["bf16"]["scalar"] * 10, 1e-9)
    k_extra = eps_z if zmax else 0.0
    e = (check_scalar(f"{tag} loss", loss, ref[0], TOL["bf16"]["scalar"], abs_tol=eps_z),
         check_scalar(f"{tag} gs", gs, ref[3], gs_tol, abs_tol=gs_abs),
         check_tensor(f"{tag} gI", gI, ref[1], "bf16", scale[0], scale[2], k_extra=k_extra, cancelling=cancelling),
         check_tensor(f"{tag} gT", gT, ref[2], "bf16", scale[1], scale[2], k_extra=k_extra, cancelling=cancelling))
    print(tag, f"loss {e[0]:.1e} gs {e[1]:.1e} gI {e[2][0]:.1e}/{e[2][1]:.2f} gT {e[3][0]:.1e}/{e[3][1]:.2f}", flush=True)


@pytest.mark.parametrize("B,d,N,s", [
    (1000, 256, 2, 14.285714),      # 500-row shares: rows and keys both padded
    (768, 128, 2, 14.285714),       # 384-row shares of a batch that is whole tiles: only the rows are padded
    (1100, 64, 1, 25.0),            # the whole batch as one ragged share (no symmetric path for it)
    (2310, 192, 3, 14.285714),      # 770-row shares: the label diagonal of ranks 1 and 2 crosses tile corners
    (264, 64, 33, 14.285714),       # 8-row shares: a single mostly empty query tile
    (1800, 512, 8, 100.0),          # 225-row shares at the clamp of the logit multiplier
    (512, 64, 512, 14.285714),      # one pair per rank
    (1, 64, 1, 14.285714),          # a batch of one pair: loss 0, no gradient
])
@pytest.mark.parametrize("path", [dl.DISCO_PATH_MATERIALIZED, dl.DISCO_PATH_FUSED], ids=["materialized", "fused"])
def test_ragged_share_matches_oracle(B, d, N, s, path):
    I, T, Ib, Tb = _inputs(B, d, 21)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    assert dl.disco_resolve_path(B, d, N, dt, path) == path
    run = GuardedRunner(Id, Td, B, d, N, dt, path)
    for r in sorted({0, N // 2, N - 1}):
        print(f"case ragged B={B} d={d} N={N} s={s} rank={r}", flush=True)
        run.rank(r, s)
        _compare(run, oc.disco_rank(I, T, s, r, N), term_scale(oc, I, T, s, r, N), f"ragged B{B} d{d} N{N} s{s:g} rank {r}")
        assert run.guards_intact()
    for r in range(N):
        run.rank(r, s, accumulate=(r > 0))
    _compare(run, oc.clip_loss_full(I, T, s), term_scale(oc, I, T, s, 0, 1), f"ragged B{B} d{d} N{N} s{s:g} accumulated")
    assert run.guards_intact()


@pytest.mark.parametrize("B,d,s,kind", [(64, 64, 14.285714, None), (1, 64, 14.285714, None), (1100, 128, 25.0, None), (1100, 64, 14.285714, None), (1000, 256, 14.285714, None), (2310, 192, 14.285714, None),
                                        (1400, 512, 100.0, "anti"), (1400, 512, 14.285714, "norms")])
def test_ragged_batch_on_the_symmetric_path(B, d, s, kind):
    """The non-decomposed loss of a batch that is not whole tiles, on the path that keeps one B x B matrix (AUTO takes
    it): padding rows and columns stay out of both directions' sums; inputs that make it hand over to the two-block
    kernels (anti-correlated positives at s = 100) go through the padding of both.  (AUTO takes this path for ragged
    batches from 512 pairs on; the smaller ones here ask for it.)"""
    I, T, Ib, Tb = _inputs(B, d, 25, kind=kind)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    assert dl.disco_resolve_path(B, d, 1, dt, dl.DISCO_PATH_SYMMETRIC) == dl.DISCO_PATH_SYMMETRIC
    zmax = abs(s) * float(np.linalg.norm(I, axis=1).max() * np.linalg.norm(T, axis=1).max())
    run = GuardedRunner(Id, Td, B, d, 1, dt, dl.DISCO_PATH_SYMMETRIC)
    print(f"case ragged symmetric B={B} d={d} s={s} {kind}", flush=True)
    run.full(s)
    ref = oc.clip_loss_full(I, T, s)
    sc = term_scale(oc, I, T, s, 0, 1)
    gsc = oc.disco_rank_gs_term_scale(I, T, s, 0, 1)
    _compare(run, ref, sc, f"ragged symmetric B{B} d{d} s{s:g} {kind}", kind is not None, gsc, zmax if kind else 0.0)
    assert run.guards_intact()
    l0, a0, t0, g0 = run.results()
    run.rank(0, s, accumulate=True)
    l1, a1, t1, g1 = run.results()
    assert l1 == pytest.approx(2 * l0, rel=1e-6) and g1 == pytest.approx(2 * g0, rel=1e-5, abs=1e-12)
    np.testing.assert_allclose(a1, 2 * a0, rtol=1e-5, atol=2e-6 * np.abs(a0).max())
    np.testing.assert_allclose(t1, 2 * t0, rtol=1e-5, atol=2e-6 * np.abs(t0).max())
    assert run.guards_intact()


@pytest.mark.parametrize("kind,s", [("big_norm_low_cos", 14.285714), ("anti", 100.0), ("zero_rows", 14.285714), ("duplicates", 100.0)])
def test_ragged_share_on_inputs_that_are_not_clip_like(kind, s):
    """The exponent reference, its repair (big_norm_low_cos loses every row total in the first pass) and the padding
    together: the padding columns must stay out of the true row maxima and the padding rows out of the flags."""
    B, d, N = 1400, 512, 2
    I, T, Ib, Tb = _inputs(B, d, 23, kind=kind)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    zmax = abs(s) * float(np.linalg.norm(I, axis=1).max() * np.linalg.norm(T, axis=1).max())
    for path in (dl.DISCO_PATH_MATERIALIZED, dl.DISCO_PATH_FUSED):
        run = GuardedRunner(Id, Td, B, d, N, dt, path)
        for r in range(N):
            print(f"case ragged {kind} s={s} rank={r} path={path}", flush=True)
            run.rank(r, s)
            _compare(run, oc.disco_rank(I, T, s, r, N), term_scale(oc, I, T, s, r, N), f"ragged {kind} s{s:g} rank {r} path {path}", True,
                     oc.disco_rank_gs_term_scale(I, T, s, r, N), zmax)
            assert run.guards_intact()


def test_ragged_share_agrees_with_the_padded_problem_rows():
    """A property that needs no oracle: a ragged call is deterministic, and its static twin (the entry point that
    allocates nothing) gives the same bits."""
    B, d, N, s = 1000, 256, 2, 14.285714
    I, T, Ib, Tb = _inputs(B, d, 22)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    run = GuardedRunner(Id, Td, B, d, N, dt, dl.DISCO_PATH_MATERIALIZED)
    run.rank(1, s)
    a = run.results()
    run.rank(1, s)
    b = run.results()
    assert a[0] == b[0] and a[3] == b[3] and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    need = dl.disco_workspace_bytes(B, d, N, dt, dl.DISCO_PATH_MATERIALIZED)
    if need <= dl.disco_static_scratch_bytes():
        st = GuardedRunner(Id, Td, B, d, N, dt, dl.DISCO_PATH_MATERIALIZED)
        dl.disco_loss_fwd_bwd_static(Id, Td, B, d, 1, N, s, dt, dl.DISCO_PATH_MATERIALIZED, 0, st.loss, st.gI, st.gT, st.gs)
        c = st.results()
        assert a[0] == c[0] and a[3] == c[3] and np.array_equal(a[1], c[1]) and np.array_equal(a[2], c[2])
        assert st.guards_intact()
