"""ctypes binding of libdisco.so: same names as include/disco.h, argument marshalling only.

Tensors are passed as torch tensors (their device pointers are taken) or as raw integer
addresses.  Nothing here computes anything.
"""
from __future__ import annotations

import ctypes
import os

# torch owns the device memory and the streams that are handed to the library, so its HIP runtime
# must be the one in the process: load it before libdisco.so, which then binds to the same
# libamdhip64 (same SONAME) instead of bringing in a second runtime with its own device context.
import torch  # noqa: F401  (import order matters)

DISCO_OK = 0
DISCO_ERR_NULL, DISCO_ERR_SHAPE, DISCO_ERR_UNSUPPORTED, DISCO_ERR_WORKSPACE, DISCO_ERR_HIP = 1, 2, 3, 4, 5
DISCO_F32, DISCO_BF16 = 0, 1
DISCO_PATH_AUTO, DISCO_PATH_NAIVE, DISCO_PATH_MATERIALIZED, DISCO_PATH_FUSED, DISCO_PATH_SYMMETRIC = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdisco.so")


class DiscoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({disco_status_string(status)})")


def library_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, f32, sz, ci = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float,
                                 ctypes.c_size_t, ctypes.c_int)
    lib.disco_resolve_path.argtypes = [i64, i64, i32, ci, ci]
    lib.disco_resolve_path.restype = ci
    lib.disco_workspace_bytes.argtypes = [i64, i64, i32, ci, ci]
    lib.disco_workspace_bytes.restype = sz
    lib.disco_loss_fwd_bwd.argtypes = [vp, vp, i64, i64, i32, i32, f32, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.disco_loss_fwd_bwd.restype = ci
    lib.disco_loss_fwd_bwd_static.argtypes = [vp, vp, i64, i64, i32, i32, f32, ci, ci, ci, vp, vp, vp, vp, vp]
    lib.disco_loss_fwd_bwd_static.restype = ci
    lib.disco_static_scratch_bytes.argtypes = []
    lib.disco_static_scratch_bytes.restype = sz
    lib.clip_loss_fwd_bwd.argtypes = [vp, vp, i64, i64, f32, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.clip_loss_fwd_bwd.restype = ci
    lib.ntxent_resolve_path.argtypes = [i64, i64, i32, ci, ci]
    lib.ntxent_resolve_path.restype = ci
    lib.ntxent_workspace_bytes.argtypes = [i64, i64, i32, ci, ci]
    lib.ntxent_workspace_bytes.restype = sz
    lib.ntxent_loss_fwd_bwd.argtypes = [vp, i64, i64, i32, i32, f32, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    lib.ntxent_loss_fwd_bwd.restype = ci
    lib.disco_set_stage_events.argtypes = [ctypes.POINTER(vp), ci]
    lib.disco_set_stage_events.restype = ci
    lib.disco_normalize_fwd.argtypes = [vp, i64, i64, ci, vp, ci, vp, vp]
    lib.disco_normalize_fwd.restype = ci
    lib.disco_normalize_bwd.argtypes = [vp, vp, ci, vp, i64, i64, vp, vp]
    lib.disco_normalize_bwd.restype = ci
    lib.disco_logit_scale_fwd.argtypes = [vp, f32, vp, vp]
    lib.disco_logit_scale_fwd.restype = ci
    lib.disco_logit_scale_bwd.argtypes = [vp, f32, vp, vp, ci, vp]
    lib.disco_logit_scale_bwd.restype = ci
    lib.disco_mfma_probe.argtypes = [ci, ci, ci, vp, vp, vp]
    lib.disco_mfma_probe.restype = ci
    lib.disco_status_string.argtypes = [ci]
    lib.disco_status_string.restype = ctypes.c_char_p
    return lib


_lib = _load()


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()       # torch tensor


def _stream_ptr(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream  # torch.cuda.Stream


def disco_status_string(status: int) -> str:
    return _lib.disco_status_string(int(status)).decode()


def disco_resolve_path(B, d, N, dtype, path) -> int:
    return _lib.disco_resolve_path(B, d, N, dtype, path)


def disco_workspace_bytes(B, d, N, dtype, path) -> int:
    return _lib.disco_workspace_bytes(B, d, N, dtype, path)


def disco_loss_fwd_bwd(I, T, B, d, rank, N, s, dtype, path, accumulate, loss, gI, gT, gs,
                       workspace, workspace_bytes, stream=None, check=True) -> int:
    st = _lib.disco_loss_fwd_bwd(_ptr(I), _ptr(T), B, d, rank, N, s, dtype, path, int(accumulate),
                                 _ptr(loss), _ptr(gI), _ptr(gT), _ptr(gs), _ptr(workspace),
                                 workspace_bytes, _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "disco_loss_fwd_bwd")
    return st


def disco_static_scratch_bytes() -> int:
    return _lib.disco_static_scratch_bytes()


def disco_loss_fwd_bwd_static(I, T, B, d, rank, N, s, dtype, path, accumulate, loss, gI, gT, gs,
                              stream=None, check=True) -> int:
    st = _lib.disco_loss_fwd_bwd_static(_ptr(I), _ptr(T), B, d, rank, N, s, dtype, path, int(accumulate),
                                        _ptr(loss), _ptr(gI), _ptr(gT), _ptr(gs), _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "disco_loss_fwd_bwd_static")
    return st


def clip_loss_fwd_bwd(I, T, B, d, s, dtype, path, loss, gI, gT, gs, workspace, workspace_bytes,
                      stream=None, check=True) -> int:
    st = _lib.clip_loss_fwd_bwd(_ptr(I), _ptr(T), B, d, s, dtype, path, _ptr(loss), _ptr(gI), _ptr(gT),
                                _ptr(gs), _ptr(workspace), workspace_bytes, _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "clip_loss_fwd_bwd")
    return st


def ntxent_resolve_path(B, d, N, dtype, path) -> int:
    return _lib.ntxent_resolve_path(B, d, N, dtype, path)


def ntxent_workspace_bytes(B, d, N, dtype, path) -> int:
    return _lib.ntxent_workspace_bytes(B, d, N, dtype, path)


def ntxent_loss_fwd_bwd(Z, B, d, rank, N, s, dtype, path, accumulate, loss, gZ, gs, workspace, workspace_bytes,
                        stream=None, check=True) -> int:
    st = _lib.ntxent_loss_fwd_bwd(_ptr(Z), B, d, rank, N, s, dtype, path, int(accumulate), _ptr(loss), _ptr(gZ),
                                  _ptr(gs), _ptr(workspace), workspace_bytes, _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "ntxent_loss_fwd_bwd")
    return st


def disco_set_stage_events(events, count: int) -> int:
    """`events`: a ctypes array of c_void_p holding hipEvent_t handles (kept alive by the caller), or None."""
    return _lib.disco_set_stage_events(events, int(count))


def disco_mfma_probe(workgroups, iters, varied, sink, clocks, stream=None, check=True) -> int:
    st = _lib.disco_mfma_probe(int(workgroups), int(iters), int(varied), _ptr(sink), _ptr(clocks), _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "disco_mfma_probe")
    return st


def disco_normalize_fwd(X, rows, d, x_dtype, U, u_dtype, inv_norm, stream=None, check=True) -> int:
    st = _lib.disco_normalize_fwd(_ptr(X), rows, d, x_dtype, _ptr(U), u_dtype, _ptr(inv_norm), _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "disco_normalize_fwd")
    return st


def disco_normalize_bwd(G, X, x_dtype, inv_norm, rows, d, DX, stream=None, check=True) -> int:
    st = _lib.disco_normalize_bwd(_ptr(G), _ptr(X), x_dtype, _ptr(inv_norm), rows, d, _ptr(DX), _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "disco_normalize_bwd")
    return st


def disco_logit_scale_fwd(theta, s_max, s, stream=None, check=True) -> int:
    st = _lib.disco_logit_scale_fwd(_ptr(theta), s_max, _ptr(s), _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "disco_logit_scale_fwd")
    return st


def disco_logit_scale_bwd(theta, s_max, gs, gtheta, accumulate=0, stream=None, check=True) -> int:
    st = _lib.disco_logit_scale_bwd(_ptr(theta), s_max, _ptr(gs), _ptr(gtheta), int(accumulate), _stream_ptr(stream))
    if check and st != DISCO_OK:
        raise DiscoError(st, "disco_logit_scale_bwd")
    return st
