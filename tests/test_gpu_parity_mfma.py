"""GPU parity of the bf16 MFMA path against the float64 oracle at sizes that span several 256x256 tiles,
several split-K slices and ranks whose diagonal sits in different tiles."""
import numpy as np
import pytest
import torch

import paper_2304_08480_amd as dl
from oracle import clip_oracle as oc
from synth import clip_pairs, f32_to_bf16_bits, bf16_bits_to_f32
from tests.gpu_util import Runner, term_scale, check_scalar, check_tensor, to_device, TOL

pytestmark = pytest.mark.gpu


def _inputs(B, d, seed, **kw):
    I, T = clip_pairs(B, d, seed, **kw)
    Ib, Tb = f32_to_bf16_bits(I), f32_to_bf16_bits(T)
    return bf16_bits_to_f32(Ib), bf16_bits_to_f32(Tb), Ib, Tb


def _compare(run, ref, scale, tag, cancelling=False, gs_scale=0.0):
    loss, gI, gT, gs = run.results()
    # d/ds: ten times the loss bar; where the inputs make its terms cancel (near-duplicate rows), the gradient bar
    # with the derived absolute part (one bf16 rounding of every softmax term: 2^-8 of the sum of term magnitudes)
    gs_tol, gs_abs = (TOL["bf16"]["frob"], 1e-9 + 2.0 ** -8 * gs_scale) if cancelling else (TOL["bf16"]["scalar"] * 10, 1e-9)
    errs = dict(
        loss=check_scalar(f"{tag} loss", loss, ref[0], TOL["bf16"]["scalar"]),
        gs=check_scalar(f"{tag} gs", gs, ref[3], gs_tol, abs_tol=gs_abs),
        gI=check_tensor(f"{tag} gI", gI, ref[1], "bf16", scale[0], scale[2], cancelling=cancelling),
        gT=check_tensor(f"{tag} gT", gT, ref[2], "bf16", scale[1], scale[2], cancelling=cancelling),
    )
    print(tag, {k: (f"{v:.2e}" if isinstance(v, float) else tuple(f"{x:.2e}" for x in v)) for k, v in errs.items()},
          flush=True)
    return loss, gI, gT, gs


@pytest.mark.parametrize("B,d,N,s,kw", [
    (1024, 256, 2, 14.285714, {}),
    (2048, 512, 4, 14.285714, {}),
    (1536, 768, 2, 14.285714, dict(hard_frac=0.1)),
    (1024, 256, 1, 100.0, dict(noise=3.5)),
    (2048, 256, 8, 100.0, {}),
    (512, 256, 2, 0.0, {}),
    (1024, 320, 2, 14.285714, {}),          # feature width a multiple of 64 only: partial column tiles
    (512, 64, 1, 14.285714, {}),
    (1024, 640, 4, 14.285714, {}),
    (3072, 192, 4, 14.285714, {}),          # 3 query tiles: super-blocks one query tile wide
    (2560, 128, 2, 25.0, {}),               # 5 query tiles, 10 key tiles
    (4096, 64, 16, 14.285714, {}),          # 256-pair shares
])
@pytest.mark.parametrize("path", [dl.DISCO_PATH_MATERIALIZED, dl.DISCO_PATH_FUSED], ids=["materialized", "fused"])
def test_mfma_path_matches_oracle(B, d, N, s, kw, path):
    I, T, Ib, Tb = _inputs(B, d, 5, **kw)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    assert dl.disco_resolve_path(B, d, N, dt, dl.DISCO_PATH_AUTO) == (dl.DISCO_PATH_MATERIALIZED if N > 1 else dl.DISCO_PATH_SYMMETRIC)
    run = Runner(Id, Td, B, d, N, dt, path)
    # near-duplicate rows, and weak positives under a sharp softmax (rows won by a negative), make gradient entries
    # differences of terms as large as the largest entries: see check_tensor
    near_ties = bool(kw.get("hard_frac")) or kw.get("noise", 0.5) > 1.0
    for r in sorted({0, N // 2, N - 1}):
        print(f"case B={B} d={d} N={N} s={s} rank={r}", flush=True)
        run.rank(r, s)
        _compare(run, oc.disco_rank(I, T, s, r, N), term_scale(oc, I, T, s, r, N),
                 f"B{B} d{d} N{N} s{s:g} rank {r}", near_ties, oc.disco_rank_gs_term_scale(I, T, s, r, N) if near_ties else 0.0)
    for r in range(N):
        run.rank(r, s, accumulate=(r > 0))
    full = oc.clip_loss_full(I, T, s)
    full_scale = term_scale(oc, I, T, s, 0, 1)
    full_gs_scale = oc.disco_rank_gs_term_scale(I, T, s, 0, 1) if near_ties else 0.0
    _compare(run, full, full_scale, f"B{B} d{d} N{N} s{s:g} accumulated", near_ties, full_gs_scale)
    run1 = Runner(Id, Td, B, d, 1, dt, path)
    run1.full(s)
    _compare(run1, full, full_scale, f"B{B} d{d} clip_loss_fwd_bwd", near_ties, full_gs_scale)
    if path == dl.DISCO_PATH_MATERIALIZED:
        # the symmetric path of the non-decomposed loss (one similarity matrix for both directions), with and
        # without accumulation into outputs that already hold something
        sym = Runner(Id, Td, B, d, 1, dt, dl.DISCO_PATH_SYMMETRIC)
        sym.full(s)
        l0, a0, t0, g0 = _compare(sym, full, full_scale, f"B{B} d{d} clip_loss_fwd_bwd symmetric", near_ties, full_gs_scale)
        sym.rank(0, s, accumulate=True)
        l1, a1, t1, g1 = sym.results()
        assert l1 == pytest.approx(2 * l0, rel=1e-6) and g1 == pytest.approx(2 * g0, rel=1e-5, abs=1e-12)
        # fp32 sums taken in another order: entries that are small residuals of larger terms move by a few ulps of those
        np.testing.assert_allclose(a1, 2 * a0, rtol=1e-5, atol=2e-6 * np.abs(a0).max())
        np.testing.assert_allclose(t1, 2 * t0, rtol=1e-5, atol=2e-6 * np.abs(t0).max())


def test_mfma_path_is_deterministic_and_accumulates():
    B, d, N, s = 1024, 256, 2, 14.285714
    I, T, Ib, Tb = _inputs(B, d, 6)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    run = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_MATERIALIZED)
    run.rank(1, s)
    l1, a1, t1, g1 = run.results()
    run.rank(1, s)
    l2, a2, t2, g2 = run.results()
    assert l1 == l2 and g1 == g2 and np.array_equal(a1, a2) and np.array_equal(t1, t2)
    run.gI.fill_(0.5); run.gT.fill_(-0.25); run.loss.fill_(2.0); run.gs.fill_(1.0)
    run.rank(1, s, accumulate=True)
    l3, a3, t3, g3 = run.results()
    assert l3 == pytest.approx(2.0 + l1, rel=1e-6) and g3 == pytest.approx(1.0 + g1, rel=1e-6)
    np.testing.assert_allclose(a3, a1 + 0.5, rtol=1e-6)
    np.testing.assert_allclose(t3, t1 - 0.25, rtol=1e-6)


def test_work_goes_to_the_stream_that_is_passed():
    # the same call on a side stream (workspace and outputs of its own) gives the identical result, and the
    # default stream is not involved: an event recorded on it before the call is complete at once
    B, d, N, s = 1024, 256, 2, 14.285714
    I, T, Ib, Tb = _inputs(B, d, 7)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    ref = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_AUTO)
    ref.rank(0, s)
    want = ref.results()
    side = torch.cuda.Stream()
    run = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_AUTO)
    torch.cuda.synchronize()
    dl.disco_loss_fwd_bwd(Id, Td, B, d, 0, N, s, dt, dl.DISCO_PATH_AUTO, 0, run.loss, run.gI, run.gT, run.gs, run.ws, run.ws_bytes, side)
    side.synchronize()
    got = (float(run.loss.item()), run.gI.cpu().numpy().astype(np.float64), run.gT.cpu().numpy().astype(np.float64), float(run.gs.item()))
    assert got[0] == want[0] and got[3] == want[3] and np.array_equal(got[1], want[1]) and np.array_equal(got[2], want[2])


def test_mfma_path_agrees_with_naive_path_on_gpu():
    # two independent kernel sets behind the same boundary
    B, d, N, s = 2048, 256, 4, 20.0
    I, T, Ib, Tb = _inputs(B, d, 8)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    fast = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_MATERIALIZED)
    slow = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_NAIVE)
    fast.rank(2, s); slow.rank(2, s)
    lf, af, tf, gf = fast.results()
    ls, as_, ts, gs_ = slow.results()
    check_scalar("loss", lf, ls, 1e-4)
    sI, sT, fl = term_scale(oc, I, T, s, 2, N)
    check_tensor("gI", af, as_, "bf16", sI, fl)
    check_tensor("gT", tf, ts, "bf16", sT, fl)


def test_fused_path_needs_less_workspace_and_matches_materialized():
    # the fused path keeps one key panel of numerators instead of the whole b x B blocks
    B, d, N, s = 4096, 256, 2, 14.285714
    I, T, Ib, Tb = _inputs(B, d, 9)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    w_mat = dl.disco_workspace_bytes(B, d, N, dt, dl.DISCO_PATH_MATERIALIZED)
    w_fus = dl.disco_workspace_bytes(B, d, N, dt, dl.DISCO_PATH_FUSED)
    b = B // N
    # two panels of B/2 keys at this size; the split-K partial buffers of the two paths may differ too
    assert abs((w_mat - w_fus) - 2 * b * (B - B // 2) * 2) <= 32 * 2 * b * d * 4 and w_fus < w_mat
    mat = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_MATERIALIZED)
    fus = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_FUSED)
    mat.rank(1, s); fus.rank(1, s)
    lm, am, tm, gm = mat.results()
    lf, af, tf, gf = fus.results()
    # same numerators, same reduction order inside a panel; the query-side sum is split differently
    assert lf == lm
    assert np.allclose(af, am, rtol=1e-4, atol=1e-10) and np.allclose(tf, tm, rtol=1e-4, atol=1e-10)
    assert gf == pytest.approx(gm, rel=1e-5)


def test_a_rank_call_can_be_captured_in_a_graph_and_replayed():
    # the library enqueues kernels only (no allocation, no memset, no synchronisation), so a caller may capture a
    # call; every replay, with eager work in between, must reproduce the eager result bit for bit
    B, d, N, s = 2048, 256, 4, 14.285714
    I, T, Ib, Tb = _inputs(B, d, 10)
    Id, Td, dt = to_device(I, T, Ib, Tb, "bf16")
    eager = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_AUTO)
    eager.rank(1, s)
    want = eager.results()
    cap = Runner(Id, Td, B, d, N, dt, dl.DISCO_PATH_AUTO)
    cap.rank(1, s)                      # warm-up outside the capture (one-time kernel attribute set-up)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cap.rank(1, s)
    for replay in range(3):
        cap.gI.fill_(float("nan")); cap.gT.fill_(float("nan")); cap.loss.fill_(float("nan")); cap.gs.fill_(float("nan"))
        eager.rank(replay % N, s)       # unrelated eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        got = cap.results()
        assert got[0] == want[0] and got[3] == want[3], f"replay {replay}"
        assert np.array_equal(got[1], want[1]) and np.array_equal(got[2], want[2]), f"replay {replay}"
