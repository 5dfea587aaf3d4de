"""moe_plan_static: the plan for callers that cannot allocate or pass a workspace (its scratch is a device
array inside the library).  Its output must be that of moe_plan, bit for bit, on two calls in a row, the
second on a smaller batch that finds the first call's leftovers in the shared scratch."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def moe():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_06055_amd as m
    m.load_library()
    return m


TABLES = ("expert_count", "rank_count", "expert_offset", "region_base", "send_idx", "row_map", "recv_count",
          "recv_offset")


def plan_both_ways(moe, cfg, M=None, me=0, stride=0, seed=0):
    from paper_2605_06055_amd.binding import MoePlan, MoeShape, _PlanStruct, _ptr
    from paper_2605_06055_amd.layer import to_device, to_host
    K = wl.make(cfg.with_(H=8), seed=seed).K
    shape = MoeShape(T=cfg.T, H=cfg.H, k=cfg.k, E=cfg.E, R=cfg.R, dtype=moe.MOE_DTYPE_BF16,
                     schedule=moe.MOE_SCHEDULE_PREFILL, rank_id=me, region_stride_rows=stride)
    kd = to_device(K)
    md = None if M is None else to_device(M)
    out = []
    for static in (False, True):
        plan = MoePlan(shape, source_count=md)
        for name in TABLES + ("status",):
            getattr(plan, name).fill_(-5)
        ps = plan.struct()
        if static:                       # no workspace at all: the entry point must not look at it
            ps = _PlanStruct(_ptr(plan.expert_count), _ptr(plan.rank_count), _ptr(plan.expert_offset),
                             _ptr(plan.region_base), _ptr(plan.send_idx), _ptr(plan.row_map), _ptr(plan.status),
                             None, 0, _ptr(md), _ptr(plan.recv_count), _ptr(plan.recv_offset))
            moe.moe_plan_static(shape, kd, ps)
        else:
            moe.moe_plan(shape, kd, ps)
        torch.cuda.synchronize()
        got = {name: to_host(getattr(plan, name)) for name in TABLES}
        got["status"] = to_host(plan.status)[:3]
        if M is None:
            got.pop("recv_count"), got.pop("recv_offset")
        out.append(got)
    for name in out[0]:
        assert np.array_equal(out[0][name], out[1][name]), name
    return out[1]


def test_static_scratch_plan_matches_moe_plan_on_two_calls(moe):
    import oracle
    big = wl.CONFIGS["skewed"].with_(T=9000)          # 72000 branches: 71 tiles, the last one ragged
    small = wl.CONFIGS["prefill"].with_(T=2000)       # 16000 branches: 16 tiles, inside the first call's leftovers
    print("[no-alloc] first call", flush=True)
    a = plan_both_ways(moe, big, seed=1)
    print("[no-alloc] second call, smaller batch", flush=True)
    b = plan_both_ways(moe, small, seed=2)
    # and both are the oracle's plan
    for cfg, got, seed in ((big, a, 1), (small, b, 2)):
        ref = oracle.plan(wl.make(cfg.with_(H=8), seed=seed).K, cfg.E, cfg.R)
        assert np.array_equal(got["row_map"][:cfg.N].reshape(cfg.T, cfg.k), ref.row_map)
        assert np.array_equal(got["expert_offset"], ref.expert_offset)
    # several source ranks and a fixed stride through the same entry point, then a batch small enough for
    # the single-launch plan (which uses no scratch) and an empty one
    M = wl.source_count_matrix(small, 8)
    plan_both_ways(moe, small, M=M, me=3, stride=9000, seed=3)
    plan_both_ways(moe, small.with_(T=700), seed=4)
    plan_both_ways(moe, small.with_(T=0), seed=5)
