"""MI355X-native decomposed CLIP contrastive loss (DisCo): thin binding over libdisco.so.

Every step of the path runs inside the HIP library; this package only marshals arguments.
There is no CPU fallback: importing `binding` fails loudly when the library is not built.
"""
from .binding import (  # noqa: F401
    DISCO_BF16,
    DISCO_ERR_HIP,
    DISCO_ERR_NULL,
    DISCO_ERR_SHAPE,
    DISCO_ERR_UNSUPPORTED,
    DISCO_ERR_WORKSPACE,
    DISCO_F32,
    DISCO_OK,
    DISCO_PATH_AUTO,
    DISCO_PATH_FUSED,
    DISCO_PATH_MATERIALIZED,
    DISCO_PATH_NAIVE,
    DISCO_PATH_SYMMETRIC,
    DiscoError,
    clip_loss_fwd_bwd,
    disco_logit_scale_bwd,
    disco_logit_scale_fwd,
    disco_loss_fwd_bwd,
    disco_mfma_probe,
    disco_loss_fwd_bwd_static,
    disco_static_scratch_bytes,
    disco_normalize_bwd,
    disco_normalize_fwd,
    disco_resolve_path,
    disco_set_stage_events,
    disco_status_string,
    disco_workspace_bytes,
    library_path,
    ntxent_loss_fwd_bwd,
    ntxent_resolve_path,
    ntxent_workspace_bytes,
)
