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


# Tolerances.  fp32 inputs: relative 1e-4.  bf16 inputs with fp32 accumulation: relative 2e-2 with an
# absolute floor of 1e-3 of the tensor's largest magnitude on gradients.  Gradient entries are of size
# 1/(2B) and smaller, so the absolute part is expressed relative to max|ref|.
TOL = {
    "f32": dict(scalar=1e-4, frob=1e-4, rel=1e-4, abs_of_max=1e-5),
    "bf16": dict(scalar=2e-3, frob=2e-2, rel=2e-2, abs_of_max=1e-3),
}


def check_scalar(name, got, ref, tol, floor=1e-30):
    err = abs(got - ref) / max(abs(ref), floor)
    assert np.isfinite(got) and err <= tol, f"{name}: got {got!r} ref {ref!r} rel err {err:.3e} > {tol}"
    return err


def check_tensor(name, got, ref, kind):
    t = TOL[kind]
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    diff = np.abs(got - ref)
    mx = np.abs(ref).max()
    fro = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    bound = t["abs_of_max"] * mx + t["rel"] * np.abs(ref)
    worst = (diff - bound).max()
    assert fro <= t["frob"], f"{name}: Frobenius rel err {fro:.3e} > {t['frob']}"
    assert worst <= 0, f"{name}: elementwise bound exceeded by {worst:.3e} (max|ref| {mx:.3e}, max diff {diff.max():.3e})"
    return fro, diff.max() / max(mx, 1e-300)
