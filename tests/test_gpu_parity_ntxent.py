"""GPU parity of the self-supervised (two-view) contrastive loss against its float64 oracle: the fp32 path on
ragged shapes, both bf16 MFMA paths on shapes of several tiles, rank counts for which a row's positive belongs to
the same rank (N = 1) and to another one (N >= 2), every rank and the accumulation over the ranks."""
import numpy as np
import pytest
import torch

import paper_2304_08480_amd as dl
from oracle import ntxent_oracle as nx
from synth import two_views, f32_to_bf16_bits, bf16_bits_to_f32
from tests.gpu_util import check_scalar, check_tensor, TOL

pytestmark = pytest.mark.gpu

PATHS = {"naive": dl.DISCO_PATH_NAIVE, "materialized": dl.DISCO_PATH_MATERIALIZED, "fused": dl.DISCO_PATH_FUSED}


class Run:
    def __init__(self, Zd, B, d, N, dt, path):
        self.Z, self.B, self.d, self.N, self.dt, self.path = Zd, B, d, N, dt, path
        self.ws_bytes = dl.ntxent_workspace_bytes(B, d, N, dt, path)
        assert self.ws_bytes > 0
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.loss = torch.full((1,), float("nan"), device="cuda")
        self.gs = torch.full((1,), float("nan"), device="cuda")
        self.gZ = torch.full((B, d), float("nan"), device="cuda")

    def rank(self, r, s, accumulate=False):
        dl.ntxent_loss_fwd_bwd(self.Z, self.B, self.d, r, self.N, s, self.dt, self.path, accumulate, self.loss, self.gZ,
                               self.gs, self.ws, self.ws_bytes, torch.cuda.current_stream())

    def results(self):
        torch.cuda.synchronize()
        return float(self.loss.item()), self.gZ.cpu().numpy().astype(np.float64), float(self.gs.item())


def _inputs(M, d, seed, dtype):
    Z = two_views(M, d, seed)
    if dtype == "bf16":
        bits = f32_to_bf16_bits(Z)
        return bf16_bits_to_f32(bits), torch.from_numpy(bits.view(np.int16)).cuda(), dl.DISCO_BF16
    return Z, torch.from_numpy(Z).cuda(), dl.DISCO_F32


def _compare(run, ref, scale, kind, tag, s, B):
    loss, gZ, gs = run.results()
    fl = 1e-13 * abs(s) / B
    e1 = check_scalar(f"{tag} loss", loss, ref[0], TOL[kind]["scalar"])
    # d/ds: ten times the loss bar, with the derived bound (one rounding of every softmax term) as the absolute part
    e2 = check_scalar(f"{tag} gs", gs, ref[2], TOL[kind]["scalar"] * 10, abs_tol=1e-9 + (2.0 ** -8 if kind == "bf16" else 1e-5) * scale[1])
    f = check_tensor(f"{tag} gZ", gZ, ref[1], kind, scale[0], fl)
    print(tag, f"loss {e1:.1e} gs {e2:.1e} gZ (fro {f[0]:.1e}, bound ratio {f[1]:.3f})", flush=True)


@pytest.mark.parametrize("M,d,N,s,dtype", [(128, 512, 4, 14.285714, "f32"), (150, 77, 3, 10.0, "f32"), (65, 33, 1, 100.0, "f32"),
                                           (96, 65, 64, 5.0, "bf16"), (4, 4, 8, 20.0, "f32"), (1, 16, 2, 3.0, "f32")])
def test_two_view_loss_fp32_path(M, d, N, s, dtype):
    B = 2 * M
    Z, Zd, dt = _inputs(M, d, 3, dtype)
    run = Run(Zd, B, d, N, dt, dl.DISCO_PATH_NAIVE)
    for r in sorted({0, N // 2, N - 1}):
        print(f"case two-view fp32 path M={M} d={d} N={N} s={s} rank={r}", flush=True)
        run.rank(r, s)
        _compare(run, nx.ntxent_rank(Z, s, r, N), nx.ntxent_rank_term_scale(Z, s, r, N), "f32", f"M{M} d{d} N{N} rank {r}", s, B)
    for r in range(N):
        run.rank(r, s, accumulate=(r > 0))
    _compare(run, nx.ntxent_full(Z, s), nx.ntxent_rank_term_scale(Z, s, 0, 1), "f32", f"M{M} d{d} N{N} accumulated", s, B)


@pytest.mark.parametrize("M,d,N,s", [(512, 256, 1, 14.285714), (512, 256, 2, 14.285714), (1024, 128, 4, 14.285714),
                                     (1536, 64, 2, 25.0), (768, 320, 6, 14.285714), (512, 128, 1, 100.0)])
@pytest.mark.parametrize("path", ["materialized", "fused"])
def test_two_view_loss_mfma_paths(path, M, d, N, s):
    B = 2 * M
    Z, Zd, dt = _inputs(M, d, 4, "bf16")
    assert dl.ntxent_resolve_path(B, d, N, dt, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_MATERIALIZED
    run = Run(Zd, B, d, N, dt, PATHS[path])
    for r in sorted({0, N // 2, N - 1}):
        print(f"case two-view {path} M={M} d={d} N={N} s={s} rank={r}", flush=True)
        run.rank(r, s)
        _compare(run, nx.ntxent_rank(Z, s, r, N), nx.ntxent_rank_term_scale(Z, s, r, N), "bf16", f"{path} M{M} d{d} N{N} rank {r}", s, B)
    for r in range(N):
        run.rank(r, s, accumulate=(r > 0))
    _compare(run, nx.ntxent_full(Z, s), nx.ntxent_rank_term_scale(Z, s, 0, 1), "bf16", f"{path} M{M} d{d} N{N} accumulated", s, B)
    # the two independent kernel sets behind the same boundary agree with each other as well
    slow = Run(Zd, B, d, N, dt, dl.DISCO_PATH_NAIVE)
    slow.rank(N - 1, s)
    run.rank(N - 1, s)
    lf, gf, sf = run.results()
    ls, gsl, ss = slow.results()
    check_scalar("loss vs fp32 path", lf, ls, 1e-4)
    check_tensor("gZ vs fp32 path", gf, gsl, "bf16", nx.ntxent_rank_term_scale(Z, s, N - 1, N)[0], 1e-13 * s / B)


@pytest.mark.parametrize("M,d,N,s", [(500, 256, 1, 14.285714),    # one ragged share holding both views: tiles straddle the views
                                     (500, 128, 2, 14.285714),    # a rank per view, 500 rows each
                                     (640, 64, 5, 25.0),          # 256-row shares of a batch whose views are not whole tiles
                                     (770, 192, 4, 14.285714),    # 385-row shares; ranks 1 and 2 meet at the view boundary
                                     (300, 64, 3, 14.285714),     # 200-row shares: rank 1 holds rows of both views
                                     (1, 64, 1, 14.285714)])      # one sample, two views: each row's only negative is nothing
@pytest.mark.parametrize("path", ["materialized", "fused"])
def test_two_view_loss_mfma_paths_on_shares_that_are_not_whole_tiles(path, M, d, N, s):
    """Shares, views and batches that are not whole 256-row tiles: operands padded in the workspace, the padding out of
    every softmax, and query tiles whose rows belong to both views (two label offsets in one tile)."""
    B = 2 * M
    Z, Zd, dt = _inputs(M, d, 6, "bf16")
    assert dl.ntxent_resolve_path(B, d, N, dt, PATHS[path]) == PATHS[path]
    run = Run(Zd, B, d, N, dt, PATHS[path])
    for r in range(N):
        print(f"case two-view ragged {path} M={M} d={d} N={N} s={s} rank={r}", flush=True)
        run.rank(r, s)
        _compare(run, nx.ntxent_rank(Z, s, r, N), nx.ntxent_rank_term_scale(Z, s, r, N), "bf16", f"ragged {path} M{M} d{d} N{N} rank {r}", s, B)
    for r in range(N):
        run.rank(r, s, accumulate=(r > 0))
    _compare(run, nx.ntxent_full(Z, s), nx.ntxent_rank_term_scale(Z, s, 0, 1), "bf16", f"ragged {path} M{M} d{d} N{N} accumulated", s, B)
