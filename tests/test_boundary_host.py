"""Host-side checks of the C ABI: the library loads, exports what include/disco.h declares, and turns
every invalid call into a status code before any GPU work (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

import paper_2304_08480_amd as dl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "disco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:disco|clip|ntxent)_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = ctypes.CDLL(dl.library_path())
    names = _declared_symbols()
    assert {"disco_loss_fwd_bwd", "clip_loss_fwd_bwd", "disco_workspace_bytes", "disco_status_string",
            "disco_resolve_path"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    for st in range(0, 6):
        assert dl.disco_status_string(st) not in ("", "unknown status")
    assert dl.disco_status_string(99) == "unknown status"


FAKE = 0x1000  # 256-aligned non-null address; never dereferenced because validation fails first


def _call(**kw):
    a = dict(I=FAKE, T=FAKE, B=256, d=512, rank=0, N=4, s=10.0, dtype=dl.DISCO_F32, path=dl.DISCO_PATH_NAIVE,
             accumulate=0, loss=FAKE, gI=FAKE, gT=FAKE, gs=FAKE, workspace=FAKE, workspace_bytes=0)
    a.update(kw)
    return dl.disco_loss_fwd_bwd(a["I"], a["T"], a["B"], a["d"], a["rank"], a["N"], a["s"], a["dtype"], a["path"],
                                 a["accumulate"], a["loss"], a["gI"], a["gT"], a["gs"], a["workspace"],
                                 a["workspace_bytes"], None, check=False)


@pytest.mark.parametrize("name", ["I", "T", "loss", "gI", "gT", "gs"])
def test_null_pointers(name):
    assert _call(**{name: None}) == dl.DISCO_ERR_NULL


@pytest.mark.parametrize("kw", [dict(B=0), dict(B=-4), dict(d=0), dict(N=0), dict(B=250, N=4), dict(rank=4),
                                dict(rank=-1), dict(B=1 << 25, N=1)])
def test_bad_shapes(kw):
    assert _call(**kw) == dl.DISCO_ERR_SHAPE


@pytest.mark.parametrize("kw", [dict(dtype=7), dict(path=9), dict(path=dl.DISCO_PATH_MATERIALIZED),  # fp32 input
                                dict(path=dl.DISCO_PATH_MATERIALIZED, dtype=dl.DISCO_BF16, d=100)])
def test_unsupported(kw):
    assert _call(**kw) == dl.DISCO_ERR_UNSUPPORTED


def test_workspace_checks():
    need = dl.disco_workspace_bytes(256, 512, 4, dl.DISCO_F32, dl.DISCO_PATH_NAIVE)
    assert need >= 2 * 64 * 256 * 4
    assert _call(workspace=None, workspace_bytes=need) == dl.DISCO_ERR_WORKSPACE
    assert _call(workspace=FAKE + 8, workspace_bytes=need) == dl.DISCO_ERR_WORKSPACE
    assert _call(workspace=FAKE, workspace_bytes=need - 1) == dl.DISCO_ERR_WORKSPACE


def test_workspace_bytes_zero_on_bad_args():
    assert dl.disco_workspace_bytes(250, 512, 4, dl.DISCO_F32, dl.DISCO_PATH_NAIVE) == 0
    assert dl.disco_workspace_bytes(256, 512, 4, 5, dl.DISCO_PATH_NAIVE) == 0
    assert dl.disco_resolve_path(250, 512, 4, dl.DISCO_F32, dl.DISCO_PATH_AUTO) == -dl.DISCO_ERR_SHAPE


def test_naive_workspace_follows_the_papers_memory_model():
    # Sec. 4.1: two b x B matrices instead of B x B -> 2 B^2 / N entries (fp32 here), plus O(b) row scalars
    for B, N in ((32768, 8), (32768, 1), (196608, 64)):
        need = dl.disco_workspace_bytes(B, 512, N, dl.DISCO_BF16, dl.DISCO_PATH_NAIVE)
        entries = 2 * (B // N) * B
        assert entries * 4 <= need <= entries * 4 + 64 * (B // N) + 4096


def test_fused_path_workspace_is_one_key_panel():
    # Sec. 4.1 counts 2 b B entries for the two logit blocks; the fused path keeps 2 b W (W <= 16384 keys)
    B, d, N = 196608, 512, 64
    b = B // N
    mat = dl.disco_workspace_bytes(B, d, N, dl.DISCO_BF16, dl.DISCO_PATH_MATERIALIZED)
    fus = dl.disco_workspace_bytes(B, d, N, dl.DISCO_BF16, dl.DISCO_PATH_FUSED)
    # the two paths may also split the query-side reduction differently (at most 32 partial tiles per block)
    assert mat >= 2 * b * B * 2 and abs((mat - fus) - 2 * b * (B - 16384) * 2) <= 32 * 2 * b * d * 4 and fus < mat
    assert dl.disco_resolve_path(B, d, N, dl.DISCO_F32, dl.DISCO_PATH_FUSED) == -dl.DISCO_ERR_UNSUPPORTED


def test_two_view_loss_argument_checks():
    def call(**kw):
        a = dict(Z=FAKE, B=256, d=64, rank=0, N=4, s=10.0, dtype=dl.DISCO_F32, path=dl.DISCO_PATH_NAIVE, loss=FAKE, gZ=FAKE,
                 gs=FAKE, ws=FAKE, ws_bytes=0)
        a.update(kw)
        return dl.ntxent_loss_fwd_bwd(a["Z"], a["B"], a["d"], a["rank"], a["N"], a["s"], a["dtype"], a["path"], 0, a["loss"],
                                      a["gZ"], a["gs"], a["ws"], a["ws_bytes"], None, check=False)

    for name in ("Z", "loss", "gZ", "gs"):
        assert call(**{name: None}) == dl.DISCO_ERR_NULL
    assert call(B=255, N=1) == dl.DISCO_ERR_SHAPE                      # two views: an even number of rows
    assert call(B=256, N=3) == dl.DISCO_ERR_SHAPE and call(rank=4) == dl.DISCO_ERR_SHAPE
    assert call() == dl.DISCO_ERR_WORKSPACE                            # valid arguments, workspace too small
    need = dl.ntxent_workspace_bytes(256, 64, 4, dl.DISCO_F32, dl.DISCO_PATH_NAIVE)
    assert need >= 64 * 256 * 4 and need < 2 * 64 * 256 * 4 + 8192     # ONE b x B block (the CLIP loss keeps two)
    # the bf16 tile paths take any share (ragged ones padded); AUTO sends tiny ragged blocks to the fp32 path
    assert dl.ntxent_resolve_path(1024, 64, 2, dl.DISCO_BF16, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_MATERIALIZED
    assert dl.ntxent_resolve_path(1000, 64, 1, dl.DISCO_BF16, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_MATERIALIZED
    assert dl.ntxent_resolve_path(1000, 64, 1, dl.DISCO_BF16, dl.DISCO_PATH_FUSED) == dl.DISCO_PATH_FUSED
    assert dl.ntxent_resolve_path(100, 64, 2, dl.DISCO_BF16, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_NAIVE
    assert dl.ntxent_resolve_path(1000, 65, 1, dl.DISCO_BF16, dl.DISCO_PATH_FUSED) == -dl.DISCO_ERR_UNSUPPORTED
    assert dl.ntxent_resolve_path(1024, 64, 1, dl.DISCO_BF16, dl.DISCO_PATH_SYMMETRIC) == -dl.DISCO_ERR_UNSUPPORTED
    assert dl.ntxent_workspace_bytes(255, 64, 1, dl.DISCO_F32, dl.DISCO_PATH_NAIVE) == 0


def test_stage_events_argument_check():
    assert dl.disco_set_stage_events(None, 0) == dl.DISCO_OK
    assert dl.disco_set_stage_events(None, -1) == dl.DISCO_ERR_SHAPE


def test_auto_falls_back_to_naive_for_fp32_and_odd_shapes():
    assert dl.disco_resolve_path(256, 512, 4, dl.DISCO_F32, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_NAIVE
    assert dl.disco_resolve_path(300, 77, 3, dl.DISCO_BF16, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_NAIVE


# ---------------------------------------------------------------- feature preparation entry points (argument checks only)
FAKE_PTR = 0x1000


def test_normalize_argument_checks():
    ok = dict(X=FAKE_PTR, rows=8, d=16, x_dtype=dl.DISCO_F32, U=FAKE_PTR, u_dtype=dl.DISCO_BF16, inv=FAKE_PTR)

    def fwd(**kw):
        a = dict(ok); a.update(kw)
        return dl.disco_normalize_fwd(a["X"], a["rows"], a["d"], a["x_dtype"], a["U"], a["u_dtype"], a["inv"], None, check=False)

    assert fwd(X=None) == dl.DISCO_ERR_NULL and fwd(U=None) == dl.DISCO_ERR_NULL and fwd(inv=None) == dl.DISCO_ERR_NULL
    assert fwd(rows=0) == dl.DISCO_ERR_SHAPE and fwd(d=-1) == dl.DISCO_ERR_SHAPE and fwd(rows=1 << 39, d=4) == dl.DISCO_ERR_SHAPE
    assert fwd(x_dtype=5) == dl.DISCO_ERR_UNSUPPORTED and fwd(u_dtype=-1) == dl.DISCO_ERR_UNSUPPORTED

    def bwd(**kw):
        a = dict(G=FAKE_PTR, X=FAKE_PTR, x_dtype=dl.DISCO_BF16, inv=FAKE_PTR, rows=8, d=16, DX=FAKE_PTR); a.update(kw)
        return dl.disco_normalize_bwd(a["G"], a["X"], a["x_dtype"], a["inv"], a["rows"], a["d"], a["DX"], None, check=False)

    for name in ("G", "X", "inv", "DX"):
        assert bwd(**{name: None}) == dl.DISCO_ERR_NULL
    assert bwd(rows=0) == dl.DISCO_ERR_SHAPE and bwd(x_dtype=9) == dl.DISCO_ERR_UNSUPPORTED


def test_logit_scale_argument_checks():
    assert dl.disco_logit_scale_fwd(None, 100.0, FAKE_PTR, None, check=False) == dl.DISCO_ERR_NULL
    assert dl.disco_logit_scale_fwd(FAKE_PTR, 0.0, FAKE_PTR, None, check=False) == dl.DISCO_ERR_SHAPE
    assert dl.disco_logit_scale_bwd(FAKE_PTR, 100.0, None, FAKE_PTR, 0, None, check=False) == dl.DISCO_ERR_NULL
    assert dl.disco_logit_scale_bwd(FAKE_PTR, float("nan"), FAKE_PTR, FAKE_PTR, 0, None, check=False) == dl.DISCO_ERR_SHAPE


def test_mfma_paths_refuse_sizes_beyond_their_32_bit_tile_offsets():
    big = 1 << 24
    assert dl.disco_resolve_path(big, 512, big // 256, dl.DISCO_BF16, dl.DISCO_PATH_MATERIALIZED) == -dl.DISCO_ERR_UNSUPPORTED
    assert dl.disco_resolve_path(big, 512, big // 256, dl.DISCO_BF16, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_NAIVE
    assert dl.disco_resolve_path(1 << 23, 512, (1 << 23) // 256, dl.DISCO_BF16, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_MATERIALIZED


def test_auto_sends_ragged_shares_to_the_tile_kernels_when_large_enough():
    dt = dl.DISCO_BF16
    assert dl.disco_resolve_path(32000, 512, 8, dt, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_MATERIALIZED
    assert dl.disco_resolve_path(1000, 256, 2, dt, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_MATERIALIZED
    assert dl.disco_resolve_path(1100, 64, 1, dt, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_SYMMETRIC
    assert dl.disco_resolve_path(264, 64, 33, dt, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_NAIVE
    assert dl.disco_resolve_path(32, 64, 4, dt, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_NAIVE
    assert dl.disco_resolve_path(1000, 100, 2, dt, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_NAIVE       # d % 64 != 0
    assert dl.disco_resolve_path(1000, 256, 1, dt, dl.DISCO_PATH_SYMMETRIC) == dl.DISCO_PATH_SYMMETRIC
    assert dl.disco_resolve_path(1000, 256, 2, dt, dl.DISCO_PATH_FUSED) == dl.DISCO_PATH_FUSED
    assert dl.disco_workspace_bytes(1000, 256, 2, dt, dl.DISCO_PATH_MATERIALIZED) > dl.disco_workspace_bytes(1024, 256, 2, dt, dl.DISCO_PATH_MATERIALIZED)


def test_bench_refuses_more_than_one_gpu():
    """Every box has one GPU: `bench.py --gpus N` with N above 1 exits with a message, before any GPU work."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
