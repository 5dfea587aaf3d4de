"""MI355X-native relay-buffer-free MoE dispatch / combine.

Thin Python binding of the C-ABI library declared in ``include/moe_rbf.h``: the functions here
have the same names as the C entry points and only marshal arguments (torch tensors -> device
pointers, the current torch stream -> hipStream_t).  Every step of the path runs in the HIP
kernels; there is no CPU or PyTorch fallback -- if the library is missing, importing the
binding's entry points raises.
"""
from .binding import (  # noqa: F401
    MOE_DTYPE_BF16, MOE_DTYPE_F32, MOE_SCHEDULE_AUTO, MOE_SCHEDULE_DECODE, MOE_SCHEDULE_PREFILL,
    MoeError, MoePlan, MoeShape, library_path, load_library, moe_combine, moe_dispatch, moe_dispatch_quant,
    moe_plan, moe_plan_static,
    moe_resolve_schedule, moe_strerror, moe_window_rows, moe_workspace_bytes,
)
