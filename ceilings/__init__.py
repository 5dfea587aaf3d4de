"""Memory-system ceilings for the two access mixes of the MoE path (measurement harness for bench.py).

Plain gather / scatter / read / write kernels in ``stream_mix.hip``, independent of the library's kernels:
what the device sustains for 8 reads : 1 write and 1 read : 8 writes of 16-byte vectors, with sequential rows
and with rows scattered over the expert blocks of a window.  Built by ``__graft_entry__.build()``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libstream_mix.so")
_lib = None


def build(out: str = LIB) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-o", out, os.path.join(HERE, "stream_mix.hip")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return out


def load():
    """Loads the built kernels (after torch's HIP runtime, like the product binding); raises if not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise ImportError(f"{LIB} not found: run __graft_entry__.build()")
        from paper_2605_06055_amd.binding import _bind_hip_runtime
        _bind_hip_runtime()
        lib = ctypes.CDLL(LIB)
        vp = ctypes.c_void_p
        lib.ceil_mix.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp, vp, ctypes.c_int, ctypes.c_int,
                                 ctypes.c_int, vp]
        lib.ceil_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int, vp]
        lib.ceil_write.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, vp]
        for f in (lib.ceil_mix, lib.ceil_read, lib.ceil_write):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


GATHER, SCATTER = 0, 1


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def mix(kind, n_per_row, src, table, dst, rows, cols, grid=0, plain=False):
    """One launch of the gather (kind 0) or scatter (kind 1) kernel; the table's entries must lie inside the
    indexed buffer (checked here, on the host, before anything is launched)."""
    indexed = src if kind == GATHER else dst
    other = dst if kind == GATHER else src
    assert table.numel() == rows * n_per_row and table.dtype.itemsize == 4
    assert indexed.numel() * indexed.element_size() >= rows * n_per_row * cols * 16
    assert other.numel() * other.element_size() >= rows * cols * 16
    rc = load().ceil_mix(kind, n_per_row, int(plain), src.data_ptr(), table.data_ptr(), dst.data_ptr(), rows, cols,
                         grid, _stream())
    if rc:
        raise RuntimeError(f"ceil_mix launch failed ({rc})")


def read(src, sink, grid=4096):
    rc = load().ceil_read(src.data_ptr(), src.numel() * src.element_size() // 16, sink.data_ptr(), grid, _stream())
    if rc:
        raise RuntimeError(f"ceil_read launch failed ({rc})")


def write(dst, grid=4096):
    rc = load().ceil_write(dst.data_ptr(), dst.numel() * dst.element_size() // 16, grid, _stream())
    if rc:
        raise RuntimeError(f"ceil_write launch failed ({rc})")
