"""MI355X-native fused token loss of the UloRL objective (arxiv 2507.19766).

The package is a thin ctypes binding over ``lib/libulorl.so`` (hand-written HIP for gfx950,
C ABI declared in ``include/ulorl.h``).  PyTorch is used for device memory and streams only;
there is no CPU or eager fallback: without the built library, or without a GPU, calls fail.
"""
from .binding import (  # noqa: F401
    F32, BF16, IS_SAIS, IS_POIS, GATE_PER_RESPONSE, GATE_GLOBAL, GATE_ALWAYS, GATE_NEVER,
    STATUS_BAD_TOKEN, STATUS_NONFINITE, STATUS_BAD_CU, STATUS_SYNC,
    LAUNCH_PER_ROW, LAUNCH_DENSE_ROWS, Launch,
    UlorlError, Params, FwdResult, lib_path, load_library, version, status_string,
    token_loss_workspace_bytes, token_loss_fwd, token_loss_bwd, token_loss_fwd_bwd, token_loss_fwd_bwd_static, init, static_scratch_bytes, row_stats,
    lmhead_workspace_bytes, lmhead_token_loss_fwd, lmhead_token_loss_bwd, gemm_tn_bf16,
    advantage_prep, segment_diagnostics, segment_pool_step,
)
from . import autograd  # noqa: F401,E402
