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
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.ceil_gather8.argtypes = [ci, ci, ci, vp, vp, vp, ci, ci, vp]
        lib.ceil_scatter8.argtypes = [ci, ci, ci, vp, vp, vp, ci, ci, vp]
        lib.ceil_write.argtypes = [ci, vp, ctypes.c_size_t, vp]
        lib.ceil_read.argtypes = [ci, vp, ctypes.c_size_t, vp, vp]
        for f in (lib.ceil_gather8, lib.ceil_scatter8, lib.ceil_read, lib.ceil_write):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check_table(table, n_rows_indexed):
    """The kernels trust the table: its entries are checked here, once, on the host."""
    assert table.dtype.itemsize == 4
    lo, hi = int(table.min().item()), int(table.max().item())
    assert 0 <= lo and hi < n_rows_indexed, "table entry outside the indexed buffer"


# forms tried for each mix: (workgroup size or table entries per workgroup, nontemporal loads, mapping)
GATHER_FORMS = [(64, True, 0), (128, True, 0), (128, True, 1), (512, True, 3)]      # mapping 3 needs cols % 64 == 0
SCATTER_FORMS = [(1, False, 1), (1, False, 2), (1, True, 1), (8, False, 0), (8, True, 0)]


def gather8(form, src, table, dst, rows, cols):
    """dst[t] = OR of the 8 rows of src named by table[8t .. 8t+8)."""
    block, nt, mapping = form
    assert table.numel() == rows * 8 and src.numel() * src.element_size() >= rows * 8 * cols * 16
    assert dst.numel() * dst.element_size() >= rows * cols * 16
    rc = load().ceil_gather8(block, int(nt), mapping, src.data_ptr(), table.data_ptr(), dst.data_ptr(), rows, cols,
                             _stream())
    if rc:
        raise RuntimeError(f"ceil_gather8 launch failed ({rc})")


def scatter8(form, src, table, dst, rows, cols):
    """dst[table[8t + j]] = src[t] for j = 0..7."""
    per_unit, nt, mapping = form
    assert table.numel() == rows * 8 and dst.numel() * dst.element_size() >= rows * 8 * cols * 16
    assert src.numel() * src.element_size() >= rows * cols * 16
    rc = load().ceil_scatter8(per_unit, int(nt), mapping, src.data_ptr(), table.data_ptr(), dst.data_ptr(), rows, cols,
                              _stream())
    if rc:
        raise RuntimeError(f"ceil_scatter8 launch failed ({rc})")


def read(src, sink, nt=True):
    rc = load().ceil_read(int(nt), src.data_ptr(), src.numel() * src.element_size() // 16, sink.data_ptr(), _stream())
    if rc:
        raise RuntimeError(f"ceil_read launch failed ({rc})")


def write(dst, nt=False):
    rc = load().ceil_write(int(nt), dst.data_ptr(), dst.numel() * dst.element_size() // 16, _stream())
    if rc:
        raise RuntimeError(f"ceil_write launch failed ({rc})")
