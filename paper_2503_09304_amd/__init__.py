"""qmoe: a priority-ordered, preemptible Mixture-of-Experts layer for AMD MI355X (gfx950).

The work is done by libqmoe.so (hand-written HIP kernels behind the C ABI of include/qmoe.h).
This package only marshals arguments; there is no CPU or PyTorch fallback, and loading fails
loudly when the library has not been built (python -m paper_2503_09304_amd.build)."""
from .binding import (  # noqa: F401
    MOE_BF16,
    MOE_CLASS_ALL,
    MOE_CLASS_BE,
    MOE_CLASS_LS,
    MOE_DONE,
    MOE_E_ARG,
    MOE_E_HIP,
    MOE_E_INCOMPLETE,
    MOE_E_STATE,
    MOE_E_WORKSPACE,
    MOE_F32,
    MOE_OK,
    MOE_W_PACKED,
    MOE_W_ROWMAJOR,
    UINT32_MAX,
    Context,
    MoeConfig,
    MoeCursor,
    MoeError,
    MoeUnit,
    MoeWeights,
    lib,
    lib_path,
    moe_last_error,
    moe_pack_weights,
    moe_plan_units,
    moe_workspace_bytes,
)
