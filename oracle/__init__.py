"""ctypes front end of the CPU oracle (``moe_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's cpu_baseline leg; never by the product package.  Arguments are numpy
arrays; bf16 tensors travel as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

_LIB_OMP = os.path.join(_HERE, "libmoe_oracle_omp.so")

BF16, F32 = 0, 1
_lib = None
_serial = _parallel = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  ``-ffp-contract=off`` keeps the compiler from fusing or
    splitting anything: the only fused multiply-adds are the explicit ``fmaf`` calls."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-mfma", "-ffp-contract=off", "-Wall", "-Wextra", "-shared",
                               "-fPIC", "-o", _LIB, _SRC, "-lm"])
    if force or not os.path.exists(_LIB_OMP) or os.path.getmtime(_LIB_OMP) < os.path.getmtime(_SRC):
        # the same file with the token loops of dispatch and combine handed to all cores (benchmark only)
        subprocess.check_call(["gcc", "-O2", "-mfma", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", "-shared",
                               "-fPIC", "-o", _LIB_OMP, _SRC, "-lm"])
    return _LIB


def _open(path):
    lib = ctypes.CDLL(path)
    for name in ("moe_ref_plan", "moe_ref_plan_multi", "moe_ref_dispatch", "moe_ref_combine", "moe_ref_combine_f64",
                 "moe_ref_expert_standin", "moe_ref_threads"):
        getattr(lib, name).restype = ctypes.c_int
    return lib


def _load():
    global _lib, _serial
    if _lib is None:
        build(force=False)
        _lib = _serial = _open(_LIB)
    return _lib


def threads() -> int:
    """Threads the loaded build hands the token loops of dispatch and combine to (1 unless all_cores())."""
    return int(_load().moe_ref_threads())


class all_cores:
    """``with oracle.all_cores():`` runs dispatch and combine of the enclosed calls on every host core
    (the OpenMP build of the same source).  For the benchmark's baseline; the tests use the serial build."""

    def __enter__(self):
        global _lib, _parallel
        _load()
        if _parallel is None:
            _parallel = _open(_LIB_OMP)
        _lib = _parallel
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = _serial
        return False


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _dtype_of(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return F32
    raise TypeError(f"storage dtype must be uint16 (bf16 bits) or float32, got {a.dtype}")


@dataclass
class Plan:
    c_exp: np.ndarray          # [E]   per-expert routed-branch counts
    c_rank: np.ndarray         # [R]   per-rank routed-branch counts
    expert_offset: np.ndarray  # [E+1] large offset o
    region_base: np.ndarray    # [R+1]
    s: np.ndarray              # [T,k] small offset
    row_map: np.ndarray        # [T,k] o[K] + s, -1 when skipped
    status: np.ndarray         # [3]   {#invalid ids, #dropped for capacity, rows of all sources >= 2^31}

    @property
    def window_rows(self) -> int:
        return int(self.region_base[-1])


def plan(K: np.ndarray, E: int, R: int, region_stride_rows: int = 0) -> Plan:
    K = np.ascontiguousarray(K, dtype=np.int32)
    T, k = K.shape
    out = Plan(np.zeros(E, np.int32), np.zeros(R, np.int32), np.zeros(E + 1, np.int32),
               np.zeros(R + 1, np.int32), np.zeros((T, k), np.int32), np.zeros((T, k), np.int32),
               np.zeros(3, np.int32))
    rc = _load().moe_ref_plan(ctypes.c_int32(T), ctypes.c_int32(k), ctypes.c_int32(E), ctypes.c_int32(R),
                              ctypes.c_int64(region_stride_rows), _p(K), _p(out.c_exp), _p(out.c_rank),
                              _p(out.expert_offset), _p(out.region_base), _p(out.s), _p(out.row_map),
                              _p(out.status))
    if rc != 0:
        raise ValueError(f"moe_ref_plan rejected the shape (rc={rc})")
    return out


@dataclass
class MultiPlan(Plan):
    o_all: np.ndarray = None         # [E,R] o_{e,r}: first row of the sub-block (expert e, source rank r)
    recv_count: np.ndarray = None    # [E]   n^exp: rows of expert e's whole block (all sources)
    recv_offset: np.ndarray = None   # [E+1] first row of expert e's whole block; [E] = end of the last block

    @property
    def window_rows(self) -> int:
        return int(max(self.region_base[-1], self.recv_offset[-1]))


def plan_multi(K: np.ndarray, M: np.ndarray, me: int, E: int, R: int, region_stride_rows: int = 0) -> MultiPlan:
    """Plan of source rank `me` when M[r,e] branches arrive from the other source ranks (row `me` of M is ignored)."""
    K = np.ascontiguousarray(K, dtype=np.int32)
    M = np.ascontiguousarray(M, dtype=np.int32)
    assert M.shape == (R, E)
    T, k = K.shape
    out = MultiPlan(np.zeros(E, np.int32), np.zeros(R, np.int32), np.zeros(E + 1, np.int32),
                    np.zeros(R + 1, np.int32), np.zeros((T, k), np.int32), np.zeros((T, k), np.int32),
                    np.zeros(3, np.int32), np.zeros((E, R), np.int32), np.zeros(E, np.int32),
                    np.zeros(E + 1, np.int32))
    rc = _load().moe_ref_plan_multi(ctypes.c_int32(T), ctypes.c_int32(k), ctypes.c_int32(E), ctypes.c_int32(R),
                                    ctypes.c_int64(region_stride_rows), ctypes.c_int32(me), _p(K), _p(M),
                                    _p(out.c_exp), _p(out.c_rank), _p(out.expert_offset), _p(out.region_base),
                                    _p(out.s), _p(out.row_map), _p(out.status), _p(out.o_all), _p(out.recv_count),
                                    _p(out.recv_offset))
    if rc != 0:
        raise ValueError(f"moe_ref_plan_multi rejected the shape (rc={rc})")
    return out


def dispatch(X: np.ndarray, row_map: np.ndarray, rows: int, fill=None) -> np.ndarray:
    """Returns the window [rows, H]; rows no branch maps to keep ``fill`` (default 0)."""
    X = np.ascontiguousarray(X)
    row_map = np.ascontiguousarray(row_map, dtype=np.int32)
    T, H = X.shape
    k = row_map.shape[1]
    window = np.zeros((rows, H), X.dtype) if fill is None else np.full((rows, H), fill, X.dtype)
    rc = _load().moe_ref_dispatch(ctypes.c_int32(T), ctypes.c_int32(H), ctypes.c_int32(k),
                                  ctypes.c_int32(X.dtype.itemsize), _p(X), _p(row_map), _p(window))
    assert rc == 0
    return window


def dispatch_quant(X: np.ndarray, row_map: np.ndarray, rows: int, fill=0):
    """Row-wise quantised dispatch: returns (window_q [rows,H] uint8 e4m3 codes, window_scale [rows] float32)."""
    X = np.ascontiguousarray(X, dtype=np.uint16)
    row_map = np.ascontiguousarray(row_map, dtype=np.int32)
    T, H = X.shape
    k = row_map.shape[1]
    wq = np.full((rows, H), fill, np.uint8)
    ws = np.full(rows, -1.0, np.float32)
    rc = _load().moe_ref_dispatch_quant(ctypes.c_int32(T), ctypes.c_int32(H), ctypes.c_int32(k), _p(X), _p(row_map),
                                        _p(wq), _p(ws))
    assert rc == 0
    return wq, ws


def f32_to_e4m3(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, np.uint8)
    _load().moe_ref_f32_to_e4m3(_p(a), _p(out), ctypes.c_int64(a.size))
    return out


def _combine(fn, Yexp, W, row_map):
    Yexp = np.ascontiguousarray(Yexp)
    W = np.ascontiguousarray(W, dtype=np.float32)
    row_map = np.ascontiguousarray(row_map, dtype=np.int32)
    T, k = row_map.shape
    H = Yexp.shape[1]
    Y = np.zeros((T, H), Yexp.dtype)
    rc = fn(ctypes.c_int32(T), ctypes.c_int32(H), ctypes.c_int32(k), ctypes.c_int32(_dtype_of(Yexp)),
            _p(Yexp), _p(W), _p(row_map), _p(Y))
    assert rc == 0
    return Y


def combine(Yexp: np.ndarray, W: np.ndarray, row_map: np.ndarray) -> np.ndarray:
    """fp32 accumulation, ascending j, one fused multiply-add per branch, one rounding."""
    return _combine(_load().moe_ref_combine, Yexp, W, row_map)


def combine_f64(Yexp: np.ndarray, W: np.ndarray, row_map: np.ndarray) -> np.ndarray:
    """The same sum carried in fp64 and rounded once."""
    return _combine(_load().moe_ref_combine_f64, Yexp, W, row_map)


def expert_standin(window: np.ndarray, K: np.ndarray, row_map: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Stand-in expert FFN: every placed row times its expert's scalar, rounded to storage."""
    window = np.ascontiguousarray(window)
    K = np.ascontiguousarray(K, dtype=np.int32)
    row_map = np.ascontiguousarray(row_map, dtype=np.int32)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    T, k = K.shape
    H = window.shape[1]
    Yexp = np.zeros_like(window)
    rc = _load().moe_ref_expert_standin(ctypes.c_int32(T), ctypes.c_int32(H), ctypes.c_int32(k),
                                        ctypes.c_int32(_dtype_of(window)), _p(K), _p(row_map), _p(scale),
                                        _p(window), _p(Yexp))
    assert rc == 0
    return Yexp


def f32_to_bf16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, np.uint16)
    _load().moe_ref_f32_to_bf16(_p(a), _p(out), ctypes.c_int64(a.size))
    return out


def f64_to_bf16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    out = np.empty(a.shape, np.uint16)
    _load().moe_ref_f64_to_bf16(_p(a), _p(out), ctypes.c_int64(a.size))
    return out


def layer(X, K, W, scale, E, R, region_stride_rows: int = 0):
    """Whole chain of Algorithm 1 with the stand-in expert: returns (plan, window, Yexp, Y)."""
    pl = plan(K, E, R, region_stride_rows)
    window = dispatch(X, pl.row_map, pl.window_rows)
    Yexp = expert_standin(window, K, pl.row_map, scale)
    Y = combine(Yexp, W, pl.row_map)
    return pl, window, Yexp, Y
