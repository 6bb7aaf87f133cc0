"""GPU parity on inputs that are NOT CLIP-like (Alg. 1's cross_entropy_loss is defined for arbitrary logits):
rows of other norms, positives that are not the row maximum or are anti-correlated, exact duplicates, zero
rows, and rows whose every logit lies far below its Cauchy-Schwarz bound (the bf16 paths take their exponent
reference from the positive pair and the row norms, so these are the inputs that stress it).  Dense against
the float64 oracle, both bf16 MFMA paths and the fp32 path, single ranks and the accumulated result."""
import numpy as np
import pytest

import paper_2304_08480_amd as dl
from oracle import clip_oracle as oc
from synth import ADVERSARIAL_KINDS, adversarial_pairs, f32_to_bf16_bits, bf16_bits_to_f32
from tests.gpu_util import Runner, term_scale, check_scalar, check_tensor, to_device, TOL

pytestmark = pytest.mark.gpu

PATHS = {"materialized": dl.DISCO_PATH_MATERIALIZED, "fused": dl.DISCO_PATH_FUSED, "naive": dl.DISCO_PATH_NAIVE}


def _zmax(I, T, s):
    """Largest logit magnitude the inputs allow (Cauchy-Schwarz)."""
    return abs(s) * float(np.linalg.norm(I, axis=1).max() * np.linalg.norm(T, axis=1).max())


def _compare(run, ref, scale, kind, tag, zmax, gs_scale):
    # a logit kept in fp32 is good to |z| 2^-24: that much absolute uncertainty in every row's cross-entropy
    # (the loss is their mean over 2B rows times the rank's share) and that much relative in every softmax term
    eps_z = zmax * 2.0 ** -22
    loss, gI, gT, gs = run.results()
    # d/ds is a gradient: it gets the gradient bar of its dtype (2e-2 for bf16 inputs), and, because the sum over
    # all pairs of G_ij S_ij cancels on these inputs (exactly, for a duplicate pair), the derived bound as its
    # absolute part: one bf16 rounding of every P_ij moves it by at most 2^-8 of the sum of the term magnitudes
    gs_tol = TOL[kind]["frob"] if kind == "bf16" else TOL[kind]["scalar"] * 10
    gs_abs = 1e-9 + ((2.0 ** -8 if kind == "bf16" else 1e-5) + eps_z) * gs_scale
    e = (check_scalar(f"{tag} loss", loss, ref[0], TOL[kind]["scalar"], abs_tol=eps_z),
         check_scalar(f"{tag} gs", gs, ref[3], gs_tol, abs_tol=gs_abs),
         check_tensor(f"{tag} gI", gI, ref[1], kind, scale[0], scale[2], k_extra=eps_z, cancelling=True),
         check_tensor(f"{tag} gT", gT, ref[2], kind, scale[1], scale[2], k_extra=eps_z, cancelling=True))
    print(tag, f"loss {e[0]:.1e} gs {e[1]:.1e} gI (fro {e[2][0]:.1e}, bound ratio {e[2][1]:.2f}) "
               f"gT (fro {e[3][0]:.1e}, bound ratio {e[3][1]:.2f})", flush=True)


@pytest.mark.parametrize("s", [14.285714, 100.0], ids=["s14", "s100"])
@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
@pytest.mark.parametrize("path", list(PATHS), ids=list(PATHS))
def test_adversarial_inputs_match_oracle(path, kind, s):
    B, d, N = 1024, 256, 2
    if path == "naive" and s > 50 and kind in ("norms", "big_norm_low_cos"):
        pytest.skip("logits of magnitude 900 to 1600: their fp32 rounding alone (|z| 2^-24) exceeds the 1e-4 bar of the fp32 path")
    I, T = adversarial_pairs(B, d, 11, kind)
    Ib, Tb = f32_to_bf16_bits(I), f32_to_bf16_bits(T)
    I, T = bf16_bits_to_f32(Ib), bf16_bits_to_f32(Tb)           # the oracle sees what the GPU reads
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    kind_tol = "f32" if path == "naive" else "bf16"             # the fp32 path rounds nothing to bf16
    run = Runner(Id, Td, B, d, N, dt, PATHS[path])
    for r in range(N):
        print(f"case {path} {kind} s={s} rank={r}", flush=True)
        run.rank(r, s)
        _compare(run, oc.disco_rank(I, T, s, r, N), term_scale(oc, I, T, s, r, N), kind_tol, f"{path} {kind} s{s:g} rank {r}",
                 _zmax(I, T, s), oc.disco_rank_gs_term_scale(I, T, s, r, N))
    for r in range(N):
        run.rank(r, s, accumulate=(r > 0))
    _compare(run, oc.clip_loss_full(I, T, s), term_scale(oc, I, T, s, 0, 1), kind_tol, f"{path} {kind} s{s:g} accumulated",
             _zmax(I, T, s), oc.disco_rank_gs_term_scale(I, T, s, 0, 1))


@pytest.mark.parametrize("s", [14.285714, 100.0], ids=["s14", "s100"])
@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
def test_adversarial_inputs_symmetric_full_loss(kind, s):
    """The symmetric path of the non-decomposed loss keeps one matrix of numerators against one reference; inputs
    whose row or column totals that loses (anti-correlated positives at s = 100, rows far below their bound) must
    be handed over to the two-block kernels inside the call and still match the oracle."""
    B, d = 1024, 256
    I, T = adversarial_pairs(B, d, 13, kind)
    Ib, Tb = f32_to_bf16_bits(I), f32_to_bf16_bits(T)
    I, T = bf16_bits_to_f32(Ib), bf16_bits_to_f32(Tb)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    run = Runner(Id, Td, B, d, 1, dt, dl.DISCO_PATH_SYMMETRIC)
    print(f"case symmetric {kind} s={s}", flush=True)
    run.full(s)
    _compare(run, oc.clip_loss_full(I, T, s), term_scale(oc, I, T, s, 0, 1), "bf16", f"symmetric {kind} s{s:g}", _zmax(I, T, s),
             oc.disco_rank_gs_term_scale(I, T, s, 0, 1))


def test_rows_far_below_their_bound_take_the_slow_path():
    """big_norm_low_cos at s = 1/0.07: the reference derived from the norms lies more than 160 (base 2) above
    every logit of every row, so the first pass loses all row totals and every query tile is redone against the
    true row maxima.  The result must match the oracle as closely as any other input does."""
    B, d, N, s, r = 1536, 512, 2, 14.285714, 1
    I, T = adversarial_pairs(B, d, 12, "big_norm_low_cos")
    Ib, Tb = f32_to_bf16_bits(I), f32_to_bf16_bits(T)
    I, T = bf16_bits_to_f32(Ib), bf16_bits_to_f32(Tb)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    # the premise: every logit of every row of the rank is at least 60 (base 2) below the bound minus 100
    z2 = s * 1.4426950408889634 * (I[r * (B // N):(r + 1) * (B // N)].astype(np.float64) @ T.T.astype(np.float64))
    bound2 = s * 1.4426950408889634 * np.linalg.norm(I, axis=1).max() * np.linalg.norm(T, axis=1).max()
    assert (z2.max(axis=1) < bound2 - 100 - 60).all()
    ref = oc.disco_rank(I, T, s, r, N)
    sc = term_scale(oc, I, T, s, r, N)
    for path in ("materialized", "fused"):
        run = Runner(Id, Td, B, d, N, dt, PATHS[path])
        run.rank(r, s)
        _compare(run, ref, sc, "bf16", f"slow path {path}", _zmax(I, T, s), oc.disco_rank_gs_term_scale(I, T, s, r, N))
