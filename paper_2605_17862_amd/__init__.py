"""MI355X-native f-OPD loss pass: a thin ctypes binding over the HIP library in csrc/."""

from .binding import (  # noqa: F401
    FOPD_BF16,
    FOPD_F32,
    FopdError,
    Hparams,
    RefreshConfig,
    RefreshState,
    fopd_freshness_score,
    fopd_loss_fwd_bwd,
    fopd_profile_enable,
    fopd_profile_read,
    fopd_profile_reset,
    fopd_refresh_decide,
    fopd_set_option,
    fopd_status_string,
    fopd_token_logprobs,
    fopd_workspace_bytes,
    fopd_workspace_init,
    fopd_workspace_status,
    library_path,
    load_library,
)
