"""GPU parity of the feature-preparation entry points against the float64 oracle, through the C ABI.

Tolerances.  Norms and scaling are fp32 on the GPU: a sum of d squares and one division, so a normalised
entry is within a few units of 2^-24 of the float64 value (bar 2e-6 relative to the row's largest entry).
A bf16 output rounds that fp32 value to nearest even; where the fp32 and float64 values straddle a rounding
boundary the stored pattern may differ by one unit in the last place, so the bar is 2^-8 relative (one ulp)
and the fraction of entries that differ at all is also bounded.  The backward is a difference of products in
fp32: bar 1e-5 of (|g| + |<g,u>| |u|) / |x| per entry.
"""
import numpy as np
import pytest
import torch

import paper_2304_08480_amd as dl
from oracle import clip_oracle as oc
from oracle import feature_prep as fp
from synth import bf16_bits_to_f32, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def _raw(rows, d, seed, scale=3.0):
    rng = np.random.default_rng(seed)
    X = (rng.normal(size=(rows, d)) * scale * rng.uniform(0.2, 4.0, size=(rows, 1))).astype(np.float32)
    return X


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("rows,d", [(1000, 512), (37, 77), (4096, 768), (5, 2051), (3, 4)])
@pytest.mark.parametrize("x_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("u_dtype", ["f32", "bf16"])
def test_normalize_forward(rows, d, x_dtype, u_dtype):
    X = _raw(rows, d, 11)
    if x_dtype == "bf16":
        bits = f32_to_bf16_bits(X)
        X = bf16_bits_to_f32(bits)                     # the exact values the GPU reads
        Xd, xt = _dev(bits.view(np.int16)), dl.DISCO_BF16
    else:
        Xd, xt = _dev(X), dl.DISCO_F32
    U = torch.empty((rows, d), dtype=torch.int16 if u_dtype == "bf16" else torch.float32, device="cuda")
    inv = torch.empty(rows, device="cuda")
    print(f"case fwd rows={rows} d={d} {x_dtype}->{u_dtype}", flush=True)
    dl.disco_normalize_fwd(Xd, rows, d, xt, U, dl.DISCO_BF16 if u_dtype == "bf16" else dl.DISCO_F32, inv, torch.cuda.current_stream())
    torch.cuda.synchronize()
    ref_U, ref_inv = fp.l2_normalize_fwd(X)
    assert np.allclose(inv.cpu().numpy(), ref_inv, rtol=2e-6)
    if u_dtype == "bf16":
        got = bf16_bits_to_f32(U.cpu().numpy().view(np.uint16)).astype(np.float64)
        assert np.all(np.abs(got - ref_U) <= 2.0 ** -8 * np.abs(ref_U) + 1e-30)
        exact = bf16_bits_to_f32(f32_to_bf16_bits(ref_U.astype(np.float32))).astype(np.float64)
        assert np.mean(got != exact) < 2e-3            # all but boundary cases are the correctly rounded value
    else:
        got = U.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref_U) <= 2e-6 * np.abs(ref_U).max(axis=1, keepdims=True))


@pytest.mark.parametrize("rows,d", [(1000, 512), (37, 77), (2048, 768), (5, 2051)])
@pytest.mark.parametrize("x_dtype", ["f32", "bf16"])
def test_normalize_backward(rows, d, x_dtype):
    X = _raw(rows, d, 12)
    G = (np.random.default_rng(13).normal(size=(rows, d)) * 1e-4).astype(np.float32)
    if x_dtype == "bf16":
        bits = f32_to_bf16_bits(X)
        X = bf16_bits_to_f32(bits)
        Xd, xt = _dev(bits.view(np.int16)), dl.DISCO_BF16
    else:
        Xd, xt = _dev(X), dl.DISCO_F32
    U = torch.empty((rows, d), dtype=torch.float32, device="cuda")
    inv = torch.empty(rows, device="cuda")
    DX = torch.full((rows, d), float("nan"), device="cuda")
    print(f"case bwd rows={rows} d={d} {x_dtype}", flush=True)
    st = torch.cuda.current_stream()
    dl.disco_normalize_fwd(Xd, rows, d, xt, U, dl.DISCO_F32, inv, st)
    dl.disco_normalize_bwd(_dev(G), Xd, xt, inv, rows, d, DX, st)
    torch.cuda.synchronize()
    ref = fp.l2_normalize_bwd(G, X)
    n = np.sqrt((X.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
    u = X / n
    scale = (np.abs(G) + np.abs((G * u).sum(axis=1, keepdims=True)) * np.abs(u)) / n
    got = DX.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert np.all(np.abs(got - ref) <= 1e-5 * scale.max(axis=1, keepdims=True) + 1e-30)
    assert np.linalg.norm(got - ref) <= 1e-5 * np.linalg.norm(ref)


def test_zero_rows_use_the_cap_and_in_place_is_allowed():
    rows, d = 6, 64
    X = _raw(rows, d, 14)
    X[2] = 0.0
    Xd = _dev(X)
    inv = torch.empty(rows, device="cuda")
    st = torch.cuda.current_stream()
    dl.disco_normalize_fwd(Xd.clone(), rows, d, dl.DISCO_F32, Xd2 := Xd.clone(), dl.DISCO_F32, inv, st)
    G = np.random.default_rng(15).normal(size=(rows, d)).astype(np.float32) * 1e-20
    Gd = _dev(G)
    dl.disco_normalize_bwd(Gd, Xd, dl.DISCO_F32, inv, rows, d, Gd, st)       # DX aliases G
    inplace = Xd.clone()
    dl.disco_normalize_fwd(inplace, rows, d, dl.DISCO_F32, inplace, dl.DISCO_F32, inv, st)   # U aliases X
    torch.cuda.synchronize()
    ref_U, ref_inv = fp.l2_normalize_fwd(X)
    assert np.all(Xd2.cpu().numpy()[2] == 0.0) and inv.cpu().numpy()[2] == pytest.approx(1e12, rel=1e-6)
    assert np.allclose(inplace.cpu().numpy(), ref_U, rtol=2e-6, atol=1e-7)
    ref = fp.l2_normalize_bwd(G, X)
    got = Gd.cpu().numpy().astype(np.float64)
    assert np.allclose(got[2], ref[2], rtol=1e-6)                              # g / eps
    assert np.allclose(got, ref, rtol=1e-4, atol=1e-5 * np.abs(ref).max())


def test_logit_scale_on_device():
    st = torch.cuda.current_stream()
    for theta, gs in [(np.log(1 / 0.07), -3.5e-3), (5.0, 1.0), (0.0, 2.0)]:
        th = torch.tensor([theta], dtype=torch.float32, device="cuda")
        s = torch.zeros(1, device="cuda")
        g = torch.full((1,), 0.25, device="cuda")
        dl.disco_logit_scale_fwd(th, 100.0, s, st)
        dl.disco_logit_scale_bwd(th, 100.0, torch.tensor([gs], dtype=torch.float32, device="cuda"), g, 1, st)
        torch.cuda.synchronize()
        assert s.item() == pytest.approx(fp.logit_scale_fwd(theta), rel=1e-6)
        assert g.item() == pytest.approx(0.25 + fp.logit_scale_bwd(theta, gs), rel=1e-6, abs=1e-12)


def test_chain_raw_features_to_raw_gradients():
    """encoder outputs -> normalise -> all ranks of the loss accumulated -> back through the normalisation,
    against the oracle chain evaluated on the bf16 features the GPU produced (so that the comparison is of
    the arithmetic, not of which way a rounding fell)."""
    B, d, N, theta = 1024, 256, 4, float(np.log(1 / 0.07))
    rng = np.random.default_rng(16)
    Xi = (rng.normal(size=(B, d)) * 2.0).astype(np.float32)
    Xt = (Xi + 0.5 * 2.0 * rng.normal(size=(B, d))).astype(np.float32)
    st = torch.cuda.current_stream()
    Xi_d, Xt_d = _dev(Xi), _dev(Xt)
    I = torch.empty((B, d), dtype=torch.int16, device="cuda"); T = torch.empty_like(I)
    inv_i = torch.empty(B, device="cuda"); inv_t = torch.empty(B, device="cuda")
    dl.disco_normalize_fwd(Xi_d, B, d, dl.DISCO_F32, I, dl.DISCO_BF16, inv_i, st)
    dl.disco_normalize_fwd(Xt_d, B, d, dl.DISCO_F32, T, dl.DISCO_BF16, inv_t, st)
    th = torch.tensor([theta], dtype=torch.float32, device="cuda"); s_d = torch.zeros(1, device="cuda")
    dl.disco_logit_scale_fwd(th, 100.0, s_d, st)
    s = float(s_d.item())
    assert dl.disco_resolve_path(B, d, N, dl.DISCO_BF16, dl.DISCO_PATH_AUTO) == dl.DISCO_PATH_MATERIALIZED
    ws_bytes = dl.disco_workspace_bytes(B, d, N, dl.DISCO_BF16, dl.DISCO_PATH_AUTO)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, device="cuda"); gs = torch.zeros(1, device="cuda")
    gI = torch.empty((B, d), device="cuda"); gT = torch.empty((B, d), device="cuda")
    for r in range(N):
        dl.disco_loss_fwd_bwd(I, T, B, d, r, N, s, dl.DISCO_BF16, dl.DISCO_PATH_AUTO, r > 0, loss, gI, gT, gs, ws, ws_bytes, st)
    dXi = torch.empty((B, d), device="cuda"); dXt = torch.empty((B, d), device="cuda")
    dl.disco_normalize_bwd(gI, Xi_d, dl.DISCO_F32, inv_i, B, d, dXi, st)
    dl.disco_normalize_bwd(gT, Xt_d, dl.DISCO_F32, inv_t, B, d, dXt, st)
    gth = torch.zeros(1, device="cuda")
    dl.disco_logit_scale_bwd(th, 100.0, gs, gth, 0, st)
    torch.cuda.synchronize()

    If = bf16_bits_to_f32(I.cpu().numpy().view(np.uint16)).astype(np.float64)
    Tf = bf16_bits_to_f32(T.cpu().numpy().view(np.uint16)).astype(np.float64)
    L, rgI, rgT, rgs = oc.clip_loss_full(If, Tf, s)
    assert loss.item() == pytest.approx(L, rel=1e-4)
    assert gth.item() == pytest.approx(fp.logit_scale_bwd(np.log(s), rgs), rel=1e-3, abs=1e-9)
    for got, g_ref, X in ((dXi, rgI, Xi), (dXt, rgT, Xt)):
        ref = fp.l2_normalize_bwd(g_ref, X)
        err = np.linalg.norm(got.cpu().numpy() - ref) / np.linalg.norm(ref)
        print("chain: relative error of the raw-feature gradient", err, flush=True)
        assert err < 2e-2
