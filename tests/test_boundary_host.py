"""Host-side behaviour of the C-ABI library that needs no GPU: it loads, exports every symbol the
header declares, and returns each documented error code from argument validation alone."""
import ctypes
import os
import re

import pytest

import paper_2605_06055_amd as moe
from paper_2605_06055_amd.binding import _PlanStruct

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "moe_rbf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = moe.load_library()
    names = declared_symbols()
    assert {"moe_plan", "moe_dispatch", "moe_combine", "moe_workspace_bytes", "moe_window_rows",
            "moe_resolve_schedule", "moe_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def shape(**kw):
    base = dict(T=64, H=256, k=4, E=16, R=4, dtype=moe.MOE_DTYPE_BF16, schedule=moe.MOE_SCHEDULE_AUTO,
                rank_id=0, region_stride_rows=0)
    base.update(kw)
    return moe.MoeShape(**base)


def code(fn, *a):
    with pytest.raises(moe.MoeError) as ei:
        fn(*a)
    return ei.value.code


def test_sizes_and_schedule():
    s = shape()
    assert moe.moe_window_rows(s) == 64 * 4
    assert moe.moe_window_rows(shape(region_stride_rows=100)) == 400
    assert moe.moe_workspace_bytes(s) % 256 == 0 and moe.moe_workspace_bytes(s) >= (16 + 1) * 4
    assert moe.moe_resolve_schedule(s) == moe.MOE_SCHEDULE_DECODE
    assert moe.moe_resolve_schedule(shape(T=1281)) == moe.MOE_SCHEDULE_PREFILL      # 5124 branches
    assert moe.moe_resolve_schedule(shape(T=1280)) == moe.MOE_SCHEDULE_DECODE       # 5120 branches
    assert moe.moe_resolve_schedule(shape(schedule=moe.MOE_SCHEDULE_PREFILL)) == moe.MOE_SCHEDULE_PREFILL
    big = shape(T=32768, H=4096, k=8, E=128, R=16)
    assert moe.moe_window_rows(big) * 4096 * 2 == 2 ** 31
    assert moe.moe_workspace_bytes(big) >= 128 * 129 * 4          # 262144 branches in tiles of 2048


@pytest.mark.parametrize("kw", [dict(T=-1), dict(H=0), dict(k=0), dict(E=0), dict(R=0), dict(E=10, R=4),
                                dict(E=2048, R=4), dict(dtype=2), dict(schedule=3), dict(rank_id=4), dict(rank_id=-1),
                                dict(region_stride_rows=-1),
                                dict(T=2000, k=8, schedule=moe.MOE_SCHEDULE_DECODE)])
def test_bad_shape(kw):
    assert code(moe.moe_window_rows, shape(**kw)) == -2
    assert code(moe.moe_workspace_bytes, shape(**kw)) == -2


def test_k_larger_than_E_is_legal():
    assert moe.moe_window_rows(shape(k=40, E=16, R=4)) == 64 * 40


def test_row_alignment():
    assert code(moe.moe_window_rows, shape(H=100)) == -3                # 200 B rows
    assert code(moe.moe_window_rows, shape(H=6, dtype=moe.MOE_DTYPE_F32)) == -3
    assert moe.moe_window_rows(shape(H=8)) == 256                        # 16 B rows are the minimum
    assert moe.moe_window_rows(shape(H=4, dtype=moe.MOE_DTYPE_F32)) == 256


def test_overflow():
    assert code(moe.moe_window_rows, shape(T=2 ** 30, k=8)) == -4
    assert code(moe.moe_window_rows, shape(region_stride_rows=2 ** 30)) == -4
    assert code(moe.moe_window_rows, shape(T=2 ** 26, k=1, H=2 ** 20)) == -4      # grid would not fit


def fake_plan(**kw):
    """Plan struct with fake (never dereferenced) 16-byte aligned device addresses."""
    vals = dict(expert_count=0x1000, rank_count=0x2000, expert_offset=0x3000, region_base=0x4000,
                send_idx=0x5000, row_map=0x6000, status=0x7000, workspace=0x8000, workspace_bytes=1 << 20,
                source_count=None, recv_count=None, recv_offset=None)
    vals.update(kw)
    return _PlanStruct(**vals)


PRE = dict(schedule=moe.MOE_SCHEDULE_PREFILL)


def test_null_pointers():
    s = shape(**PRE)
    assert code(moe.moe_plan, s, None, fake_plan(), 0) == -1
    assert code(moe.moe_plan, s, 0x100, fake_plan(row_map=None), 0) == -1
    assert code(moe.moe_plan, s, 0x100, fake_plan(expert_count=None), 0) == -1
    assert code(moe.moe_plan, s, 0x100, fake_plan(status=None), 0) == -1
    assert code(moe.moe_dispatch, s, None, None, fake_plan(), 0x100, 0) == -1
    assert code(moe.moe_dispatch, s, 0x100, None, fake_plan(), None, 0) == -1
    assert code(moe.moe_dispatch, shape(), 0x100, None, fake_plan(), 0x200, 0) == -1     # decode needs ids
    assert code(moe.moe_dispatch, shape(), 0x100, 0x300, fake_plan(rank_count=None), 0x200, 0) == -1
    assert code(moe.moe_combine, s, None, 0x100, fake_plan(), 0x200, 0) == -1
    assert code(moe.moe_combine, s, 0x100, None, fake_plan(), 0x200, 0) == -1
    assert code(moe.moe_combine, s, 0x100, 0x200, fake_plan(), None, 0) == -1
    assert code(moe.moe_combine, s, 0x100, 0x200, fake_plan(row_map=None), 0x300, 0) == -1
    lib = moe.load_library()
    assert lib.moe_plan(ctypes.byref(s), 0x100, None, None) == -1
    assert lib.moe_window_rows(None, ctypes.byref(ctypes.c_int64())) == -1
    assert lib.moe_window_rows(ctypes.byref(s), None) == -1


def test_pointer_alignment():
    s = shape(**PRE)
    assert code(moe.moe_plan, s, 0x104, fake_plan(), 0) == -3
    assert code(moe.moe_plan, s, 0x100, fake_plan(row_map=0x6004), 0) == -3
    assert code(moe.moe_plan, s, 0x100, fake_plan(send_idx=0x5008), 0) == -3
    assert code(moe.moe_plan, shape(T=4000, **PRE), 0x100, fake_plan(workspace=0x8001), 0) == -3
    assert code(moe.moe_plan, s, 0x100, fake_plan(source_count=0x9004), 0) == -3
    assert code(moe.moe_plan, s, 0x100, fake_plan(recv_offset=0x9008), 0) == -3
    assert code(moe.moe_plan, s, 0x100, fake_plan(prefetch=0x9008, prefetch_bytes=64), 0) == -3
    assert code(moe.moe_plan, s, 0x100, fake_plan(prefetch=0x9000, prefetch_bytes=40), 0) == -3
    assert code(moe.moe_plan_static, s, 0x100, fake_plan(prefetch=0x9004, prefetch_bytes=64), 0) == -3
    assert code(moe.moe_dispatch, s, 0x108, None, fake_plan(), 0x200, 0) == -3
    assert code(moe.moe_dispatch, s, 0x100, None, fake_plan(), 0x202, 0) == -3
    assert code(moe.moe_combine, s, 0x100, 0x204, fake_plan(), 0x300, 0) == -3
    assert code(moe.moe_combine, s, 0x100, 0x200, fake_plan(), 0x308, 0) == -3


def test_workspace():
    # batches above 12288 branches are planned in two launches that hand tile histograms over in the workspace
    s = shape(T=4000, **PRE)
    need = moe.moe_workspace_bytes(s)
    assert need >= 16 * (16 + 1) * 4
    assert code(moe.moe_plan, s, 0x100, fake_plan(workspace=None), 0) == -5
    assert code(moe.moe_plan, s, 0x100, fake_plan(workspace_bytes=need - 1), 0) == -5
    assert code(moe.moe_plan, s, 0x100, fake_plan(workspace=0x8008, workspace_bytes=need), 0) == -3


def test_static_scratch_plan_limits():
    """moe_plan_static ignores the workspace fields and rejects shapes whose tile histograms exceed its
    fixed device array (1 MiB), on the host, like every other argument error."""
    big_e = shape(T=80000, k=8, E=1024, R=64, **PRE)          # 640000 branches -> 313 tiles x 1025 words
    assert moe.moe_workspace_bytes(big_e) > (1 << 20)
    assert code(moe.moe_plan_static, big_e, 0x100, fake_plan(workspace=None, workspace_bytes=0), 0) == -5
    s = shape(T=4000, **PRE)
    assert code(moe.moe_plan_static, s, None, fake_plan(workspace=None, workspace_bytes=0), 0) == -1
    assert code(moe.moe_plan_static, s, 0x104, fake_plan(workspace=None, workspace_bytes=0), 0) == -3
    assert code(moe.moe_plan_static, shape(E=10, **PRE), 0x100, fake_plan(), 0) == -2


def test_overlapping_buffers():
    """x / window and y / expert_out must not share a byte; the extents are known on the host."""
    s = shape(**PRE)                                   # T=64, H=256 bf16: x and y are 32768 B, the window 131072 B
    xb, wb = 64 * 256 * 2, 64 * 4 * 256 * 2
    base = 0x100000
    for x, win in ((base, base), (base, base + xb - 16), (base + wb - 16, base), (base + 4096, base)):
        assert code(moe.moe_dispatch, s, x, None, fake_plan(), win, 0) == -7, (x, win)
        assert code(moe.moe_combine, s, win, 0x100, fake_plan(), x, 0) == -7, (x, win)
    # fixed stride: the window extent is R * stride rows
    wide = shape(region_stride_rows=1000, **PRE)
    assert code(moe.moe_dispatch, wide, base + 4 * 1000 * 512 - 16, None, fake_plan(), base, 0) == -7
    # quantised dispatch: codes, scales and x are three separate ranges
    assert code(moe.moe_dispatch_quant, s, base, None, fake_plan(), base + 16, 0x900000, 0) == -7
    assert code(moe.moe_dispatch_quant, s, base, None, fake_plan(), 0x900000, base + xb - 16, 0) == -7
    assert code(moe.moe_dispatch_quant, s, base, None, fake_plan(), 0x900000, 0x900000 + 256, 0) == -7


def test_empty_prefill_dispatch_and_combine_are_noops():
    s = shape(T=0, **PRE)
    moe.moe_dispatch(s, None, None, fake_plan(), None, 0)          # returns OK without any launch
    moe.moe_combine(s, None, None, fake_plan(), None, 0)


def test_quantised_dispatch_validation():
    s = shape(**PRE)
    assert code(moe.moe_dispatch_quant, shape(dtype=moe.MOE_DTYPE_F32, **PRE), 0x100, None, fake_plan(), 0x200,
                0x300, 0) == -2                                                     # x must be bf16
    assert code(moe.moe_dispatch_quant, shape(H=40000, **PRE), 0x100, None, fake_plan(), 0x200, 0x300, 0) == -2
    assert code(moe.moe_dispatch_quant, s, 0x100, None, fake_plan(), None, 0x300, 0) == -1
    assert code(moe.moe_dispatch_quant, s, 0x100, None, fake_plan(), 0x200, None, 0) == -1
    assert code(moe.moe_dispatch_quant, s, 0x100, None, fake_plan(), 0x204, 0x300, 0) == -3
    assert code(moe.moe_dispatch_quant, shape(), 0x100, None, fake_plan(), 0x200, 0x300, 0) == -1    # decode needs ids


def test_strerror():
    texts = {moe.moe_strerror(c) for c in range(0, -8, -1)}
    assert len(texts) == 8 and moe.moe_strerror(-99) == "unknown status"
