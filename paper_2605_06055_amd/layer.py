"""Device buffers of one MoE layer's dispatch/combine plus the three calls in order.

Memory plumbing only: torch allocates the tensors and provides the stream; every step of the
path runs in the HIP library through the binding.
"""
from __future__ import annotations

import numpy as np

from . import binding as B


def to_device(a: np.ndarray, device="cuda"):
    """numpy -> torch on the GPU; uint16 arrays are bf16 bit patterns."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def to_host(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class MoeLayer:
    """Buffers for shape (T,H,k,E,R): plan state, window, expert_out, Y."""

    def __init__(self, T, H, k, E, R, dtype=B.MOE_DTYPE_BF16, schedule=B.MOE_SCHEDULE_AUTO,
                 region_stride_rows=0, device="cuda", separate_expert_out=True, source_count=None, rank_id=0,
                 window_rows=None):
        import torch
        self.shape = B.MoeShape(T=T, H=H, k=k, E=E, R=R, dtype=dtype, schedule=schedule, rank_id=rank_id,
                                region_stride_rows=region_stride_rows)
        self.torch_dtype = torch.bfloat16 if dtype == B.MOE_DTYPE_BF16 else torch.float32
        # with several source ranks the caller, who holds the count matrix, sizes tight windows
        self.rows = B.moe_window_rows(self.shape) if window_rows is None else window_rows
        self.schedule = B.moe_resolve_schedule(self.shape)
        self.plan = B.MoePlan(self.shape, device=device, source_count=source_count)
        self._plan_struct = self.plan.struct()
        self.prefetch_x = False
        self.window = torch.empty((max(self.rows, 1), H), dtype=self.torch_dtype, device=device)
        self.expert_out = (torch.empty_like(self.window) if separate_expert_out else self.window)
        self.y = torch.empty((max(T, 1), H), dtype=self.torch_dtype, device=device)

    def dispatch(self, x, topk_idx, stream=None):
        """Plan (prefill schedule only) + dispatch.  With ``prefetch_x`` set the plan is told to pull x into the
        caches while it runs (moe_plan_t.prefetch)."""
        if self.schedule == B.MOE_SCHEDULE_PREFILL:
            if self.prefetch_x:
                self._plan_struct.prefetch = B._ptr(x)
                self._plan_struct.prefetch_bytes = x.numel() * x.element_size()
            B.moe_plan(self.shape, topk_idx, self._plan_struct, stream)
        B.moe_dispatch(self.shape, x, topk_idx, self._plan_struct, self.window, stream)

    def combine(self, topk_w, stream=None):
        B.moe_combine(self.shape, self.expert_out, topk_w, self._plan_struct, self.y, stream)

    def bind(self, x, topk_idx, topk_w, stream=None):
        """Pre-marshalled calls for a serving loop that re-runs the layer on the same buffers: returns
        (dispatch, combine) closures whose ctypes arguments were converted once.  The stream is the one
        current at bind time unless given.  (Per-call marshalling costs about 7 us in Python, more than
        a decode kernel takes.)"""
        import ctypes
        lib = B.load_library()
        vp = ctypes.c_void_p
        shp, ps = ctypes.byref(self.shape), ctypes.byref(self._plan_struct)
        st = vp(B._stream(stream))
        xp, kp, wp = vp(B._ptr(x)), vp(B._ptr(topk_idx)), vp(B._ptr(topk_w))
        win, eo, yp = vp(B._ptr(self.window)), vp(B._ptr(self.expert_out)), vp(B._ptr(self.y))
        self._bound_keepalive = (x, topk_idx, topk_w)
        prefill = self.schedule == B.MOE_SCHEDULE_PREFILL
        plan_fn, dispatch_fn, combine_fn = lib.moe_plan, lib.moe_dispatch, lib.moe_combine

        def dispatch():
            if prefill:
                rc = plan_fn(shp, kp, ps, st)
                if rc:
                    raise B.MoeError(rc, "moe_plan")
            rc = dispatch_fn(shp, xp, kp, ps, win, st)
            if rc:
                raise B.MoeError(rc, "moe_dispatch")

        def combine():
            rc = combine_fn(shp, eo, wp, ps, yp, st)
            if rc:
                raise B.MoeError(rc, "moe_combine")

        return dispatch, combine
