"""MI355X (gfx950) library for the per-token hot path of a group-based RL update.

The compute lives in hand-written HIP kernels behind a C ABI (include/aero.h, built into
libaero_hip.so next to this file).  This package is the thin Python binding: it marshals
torch tensors (device memory and streams only) into pointers and sizes.  There is no CPU
fallback: importing the binding without the built library raises.
"""
from .binding import (  # noqa: F401
    AdvParams,
    AeroError,
    aero_group_advantage,
    aero_grpo_loss_bwd,
    aero_grpo_loss_bwd_noalloc,
    aero_lmhead_logprob_fused,
    aero_logprob_fwd,
    aero_workspace_bytes,
    library_path,
    AERO_F32,
    AERO_BF16,
    AERO_F16,
    AERO_F8E4M3,
    AERO_ROW_PADDING,
    AERO_ROW_UNTOUCHED,
)
