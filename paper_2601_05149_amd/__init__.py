"""libmulo: the MuLo-SD parallel verification step for one MI355X (gfx950).

The package holds the HIP sources (csrc/), the in-tree build script and a thin
ctypes binding whose functions carry the names of the C ABI (include/mulo.h).
"""
from .binding import (  # noqa: F401
    MULO_ACCEPT_RATIO, MULO_ACCEPT_TAU, MULO_BF16, MULO_F32, MULO_OK, Ctx, KV, ModelCfg, MuloError, StepParams, Weights, alloc_kv, load_library,
    make_cfg, make_params, mulo_accept_local_resample, mulo_accept_local_resample_static, mulo_create, mulo_destroy, mulo_upsample_draft,
    mulo_profile, mulo_profile_read, mulo_rejection_islands, mulo_resample_islands, mulo_resample_sequential, mulo_verify_forward, mulo_verify_step, mulo_workspace_read, status_string,
    MULO_WS_ATTN, MULO_WS_FFN, MULO_WS_NORMED, MULO_WS_Q, MULO_WS_RESIDUAL)
