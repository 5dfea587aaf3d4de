"""ctypes binding of libmoe_rbf.so (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

MOE_DTYPE_BF16, MOE_DTYPE_F32 = 0, 1
MOE_SCHEDULE_AUTO, MOE_SCHEDULE_PREFILL, MOE_SCHEDULE_DECODE = 0, 1, 2

_PKG = os.path.dirname(os.path.abspath(__file__))
_lib = None


class MoeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = f" [{load_library().moe_last_launch_error().decode()}]" if code == -6 else ""
        super().__init__(f"{where}: {moe_strerror(code)} ({code}){detail}")


class MoeShape(ctypes.Structure):
    """Mirror of ``moe_shape``."""
    _fields_ = [("T", ctypes.c_int32), ("H", ctypes.c_int32), ("k", ctypes.c_int32), ("E", ctypes.c_int32),
                ("R", ctypes.c_int32), ("dtype", ctypes.c_int32), ("schedule", ctypes.c_int32),
                ("rank_id", ctypes.c_int32), ("region_stride_rows", ctypes.c_int64)]


class _PlanStruct(ctypes.Structure):
    """Mirror of ``moe_plan_t``."""
    _fields_ = [("expert_count", ctypes.c_void_p), ("rank_count", ctypes.c_void_p),
                ("expert_offset", ctypes.c_void_p), ("region_base", ctypes.c_void_p),
                ("send_idx", ctypes.c_void_p), ("row_map", ctypes.c_void_p), ("status", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("source_count", ctypes.c_void_p), ("recv_count", ctypes.c_void_p), ("recv_offset", ctypes.c_void_p),
                ("dispatch_order", ctypes.c_void_p), ("prefetch", ctypes.c_void_p),
                ("prefetch_bytes", ctypes.c_size_t)]


def library_path() -> str:
    return os.environ.get("MOE_RBF_LIB", os.path.join(_PKG, "libmoe_rbf.so"))


def _bind_hip_runtime() -> None:
    """libmoe_rbf.so needs the HIP runtime by soname.  PyTorch ships its own libamdhip64 (same soname, not
    /opt/rocm's file); if the library were opened first it would pull in /opt/rocm's copy and torch
    would then load a second runtime whose streams and devices are not the library's.  Loading torch's
    copy first makes the dynamic loader reuse it for the library: one runtime per process."""
    try:
        import torch
        cand = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    except ImportError:
        cand = ""
    if os.path.exists(cand):
        ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)


def load_library():
    """Loads the built HIP library; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} not found: build it with `python -m paper_2605_06055_amd.build` "
                              "(or __graft_entry__.build()); this package has no CPU fallback")
        _bind_hip_runtime()
        lib = ctypes.CDLL(path)
        vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
        shp, plp = ctypes.POINTER(MoeShape), ctypes.POINTER(_PlanStruct)
        lib.moe_workspace_bytes.argtypes = [shp, ctypes.POINTER(ctypes.c_size_t)]
        lib.moe_window_rows.argtypes = [shp, ctypes.POINTER(ctypes.c_int64)]
        lib.moe_resolve_schedule.argtypes = [shp, i32p]
        lib.moe_plan.argtypes = [shp, vp, plp, vp]
        lib.moe_plan_static.argtypes = [shp, vp, plp, vp]
        lib.moe_dispatch.argtypes = [shp, vp, vp, plp, vp, vp]
        lib.moe_combine.argtypes = [shp, vp, vp, plp, vp, vp]
        lib.moe_dispatch_quant.argtypes = [shp, vp, vp, plp, vp, vp, vp]
        lib.moe_strerror.argtypes = [ctypes.c_int]
        lib.moe_strerror.restype = ctypes.c_char_p
        lib.moe_last_launch_error.argtypes = []
        lib.moe_last_launch_error.restype = ctypes.c_char_p
        for f in ("moe_workspace_bytes", "moe_window_rows", "moe_resolve_schedule", "moe_plan", "moe_plan_static",
                  "moe_dispatch",
                  "moe_dispatch_quant", "moe_combine"):
            getattr(lib, f).restype = ctypes.c_int
        _lib = lib
    return _lib


def moe_strerror(code: int) -> str:
    return load_library().moe_strerror(code).decode()


def _check(code: int, where: str) -> None:
    if code != 0:
        raise MoeError(code, where)


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (None stays NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors must be dense row-major"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def moe_workspace_bytes(shape: MoeShape) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().moe_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)), "moe_workspace_bytes")
    return out.value


def moe_window_rows(shape: MoeShape) -> int:
    out = ctypes.c_int64(0)
    _check(load_library().moe_window_rows(ctypes.byref(shape), ctypes.byref(out)), "moe_window_rows")
    return out.value


def moe_resolve_schedule(shape: MoeShape) -> int:
    out = ctypes.c_int32(0)
    _check(load_library().moe_resolve_schedule(ctypes.byref(shape), ctypes.byref(out)), "moe_resolve_schedule")
    return out.value


class MoePlan:
    """Device buffers of ``moe_plan_t`` held as torch tensors (memory plumbing only)."""

    def __init__(self, shape: MoeShape, device="cuda", with_send_idx: bool = True, source_count=None,
                 with_order: bool = True):
        import torch
        N = shape.T * shape.k
        i32 = dict(dtype=torch.int32, device=device)
        self.expert_count = torch.empty(shape.E, **i32)
        self.rank_count = torch.empty(shape.R, **i32)
        self.expert_offset = torch.empty(shape.E + 1, **i32)
        self.region_base = torch.empty(shape.R + 1, **i32)
        self.send_idx = torch.empty(max(N, 1), **i32) if with_send_idx else None
        self.row_map = torch.empty(max(N, 1), **i32)
        self.status = torch.empty(4, **i32)
        self.workspace = torch.empty(moe_workspace_bytes(shape), dtype=torch.uint8, device=device)
        self.source_count = source_count          # [R,E] int32 counts of the other source ranks, or None
        self.recv_count = torch.empty(shape.E, **i32)
        self.recv_offset = torch.empty(shape.E + 1, **i32)
        self.dispatch_order = torch.empty(2 * max(N, 1), **i32) if with_order else None
        self.prefetch = None                      # tensor that moe_plan should pull into the caches (normally x), or None

    def struct(self) -> _PlanStruct:
        return _PlanStruct(_ptr(self.expert_count), _ptr(self.rank_count), _ptr(self.expert_offset),
                           _ptr(self.region_base), _ptr(self.send_idx), _ptr(self.row_map), _ptr(self.status),
                           _ptr(self.workspace), self.workspace.numel(), _ptr(self.source_count),
                           _ptr(self.recv_count), _ptr(self.recv_offset), _ptr(self.dispatch_order),
                           _ptr(self.prefetch),
                           0 if self.prefetch is None else self.prefetch.numel() * self.prefetch.element_size())


def _plan_struct(plan) -> _PlanStruct:
    return plan.struct() if isinstance(plan, MoePlan) else plan


def moe_plan(shape: MoeShape, topk_idx, plan, stream=None) -> None:
    ps = _plan_struct(plan)
    _check(load_library().moe_plan(ctypes.byref(shape), _ptr(topk_idx), ctypes.byref(ps), _stream(stream)),
           "moe_plan")


def moe_plan_static(shape: MoeShape, topk_idx, plan, stream=None) -> None:
    ps = _plan_struct(plan)
    _check(load_library().moe_plan_static(ctypes.byref(shape), _ptr(topk_idx), ctypes.byref(ps), _stream(stream)),
           "moe_plan_static")


def moe_dispatch(shape: MoeShape, x, topk_idx, plan, window, stream=None) -> None:
    ps = _plan_struct(plan)
    _check(load_library().moe_dispatch(ctypes.byref(shape), _ptr(x), _ptr(topk_idx), ctypes.byref(ps),
                                       _ptr(window), _stream(stream)), "moe_dispatch")


def moe_dispatch_quant(shape: MoeShape, x, topk_idx, plan, window_q, window_scale, stream=None) -> None:
    ps = _plan_struct(plan)
    _check(load_library().moe_dispatch_quant(ctypes.byref(shape), _ptr(x), _ptr(topk_idx), ctypes.byref(ps),
                                             _ptr(window_q), _ptr(window_scale), _stream(stream)),
           "moe_dispatch_quant")


def moe_combine(shape: MoeShape, expert_out, topk_w, plan, y, stream=None) -> None:
    ps = _plan_struct(plan)
    _check(load_library().moe_combine(ctypes.byref(shape), _ptr(expert_out), _ptr(topk_w), ctypes.byref(ps),
                                      _ptr(y), _stream(stream)), "moe_combine")
