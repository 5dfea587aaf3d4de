"""Parity of the HIP path against the CPU oracle, element by element, through the C-ABI.

Bar: counts, offsets, small offsets, row map and every dispatched window byte bit-exact;
combine within 1 bf16 ulp (fp32 storage: bit-exact up to the same bound in fp32 ulps), with the
fp32 accumulate / ascending-j / fused-multiply-add decision taken in the same precision on both sides.
"""
import os

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def moe():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_06055_amd as m
    m.load_library()          # raises if the HIP library was not built: there is no fallback
    return m


def ordered_bits(a: np.ndarray) -> np.ndarray:
    """Monotone integer image of bf16 (uint16) or fp32 bit patterns."""
    if a.dtype == np.uint16:
        b = a.astype(np.int64)
        return np.where(b & 0x8000, 0x8000 - b, b)
    b = a.view(np.uint32).astype(np.int64)
    return np.where(b & 0x80000000, 0x80000000 - b, b)


def max_ulp(a, b):
    return int(np.abs(ordered_bits(a) - ordered_bits(b)).max()) if a.size else 0


SENTINEL = {np.dtype(np.uint16): 0x7B7B, np.dtype(np.float32): np.float32(-1234.5)}


def run_case(moe, X, K, W, scale, E, R, schedule, stride=0, label=""):
    """One full layer on the GPU through the C-ABI, compared with the oracle.  Returns GPU outputs."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    T, H = X.shape
    k = K.shape[1]
    dtype = moe.MOE_DTYPE_BF16 if X.dtype == np.uint16 else moe.MOE_DTYPE_F32
    print(f"[case] {label} T={T} H={H} k={k} E={E} R={R} dtype={dtype} schedule={schedule} stride={stride}",
          flush=True)
    ref = oracle.plan(K, E, R, stride)
    layer = MoeLayer(T, H, k, E, R, dtype=dtype, schedule=schedule, region_stride_rows=stride)
    fill = SENTINEL[X.dtype]
    layer.window.copy_(to_device(np.full(tuple(layer.window.shape), fill, X.dtype)))
    for t in (layer.plan.expert_count, layer.plan.rank_count, layer.plan.expert_offset, layer.plan.region_base,
              layer.plan.send_idx, layer.plan.row_map, layer.plan.status):
        t.fill_(-7)
    xd = to_device(X) if T else torch.empty((1, H), dtype=layer.torch_dtype, device="cuda")
    kd = to_device(K) if T else torch.empty((1, k), dtype=torch.int32, device="cuda")
    wd = to_device(W) if T else torch.empty((1, k), dtype=torch.float32, device="cuda")
    if layer.schedule == moe.MOE_SCHEDULE_PREFILL:
        # the row map is checked on the host before any payload is moved with it
        moe.moe_plan(layer.shape, kd, layer.plan)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(layer.plan.row_map)[:T * k].reshape(T, k), ref.row_map), "row_map (plan only)"
    layer.dispatch(xd, kd)
    torch.cuda.synchronize()

    p = layer.plan
    N = T * k
    got = dict(c_exp=to_host(p.expert_count), c_rank=to_host(p.rank_count), expert_offset=to_host(p.expert_offset),
               region_base=to_host(p.region_base), s=to_host(p.send_idx)[:N].reshape(T, k),
               row_map=to_host(p.row_map)[:N].reshape(T, k), status=to_host(p.status)[:3])
    assert np.array_equal(got["c_exp"], ref.c_exp), "expert_count"
    assert np.array_equal(got["c_rank"], ref.c_rank), "rank_count"
    assert np.array_equal(got["expert_offset"], ref.expert_offset), "expert_offset"
    assert np.array_equal(got["region_base"], ref.region_base), "region_base"
    assert np.array_equal(got["s"], ref.s), "send_idx"
    assert np.array_equal(got["row_map"], ref.row_map), "row_map"
    assert np.array_equal(got["status"], ref.status), "status"

    rows = moe.moe_window_rows(layer.shape)
    assert rows == (T * k if stride == 0 else R * stride) and ref.window_rows <= rows
    ref_window = oracle.dispatch(X, ref.row_map, rows, fill=fill)
    got_window = to_host(layer.window)[:rows]
    assert got_window.tobytes() == ref_window.tobytes(), "window bytes"

    # expert stand-in computed once on the CPU from the (bit-identical) window and used by both sides
    Yexp = oracle.expert_standin(ref_window, K, ref.row_map, scale)
    if rows:
        layer.expert_out[:rows].copy_(to_device(Yexp))
    layer.y.copy_(to_device(np.full(tuple(layer.y.shape), fill, X.dtype)))
    layer.combine(wd)
    torch.cuda.synchronize()
    got_Y = to_host(layer.y)[:T]
    ref_Y = oracle.combine(Yexp, W, ref.row_map)
    nan_ref = np.isnan(wl.bf16_bits_to_f32(ref_Y)) if ref_Y.dtype == np.uint16 else np.isnan(ref_Y)
    nan_got = np.isnan(wl.bf16_bits_to_f32(got_Y)) if got_Y.dtype == np.uint16 else np.isnan(got_Y)
    assert np.array_equal(nan_ref, nan_got)
    d = max_ulp(got_Y[~nan_ref], ref_Y[~nan_ref])
    exact = np.count_nonzero(got_Y != ref_Y)
    print(f"       combine: max ulp distance {d}, {exact} of {got_Y.size} elements differ", flush=True)
    assert d <= 1, f"combine differs from the oracle by {d} ulp"
    got["window"], got["Y"] = got_window, got_Y
    return got


def run_workload(moe, cfg, schedule, stride=0):
    w = wl.make(cfg)
    return run_case(moe, w.X, w.K, w.W, w.scale, cfg.E, cfg.R, schedule, stride, label=cfg.name)


# --------------------------------------------------------------------------- the named configurations

def test_tiny_both_schedules(moe):
    a = run_workload(moe, wl.CONFIGS["tiny"], moe.MOE_SCHEDULE_PREFILL)
    b = run_workload(moe, wl.CONFIGS["tiny"], moe.MOE_SCHEDULE_DECODE)
    for key in a:
        assert np.array_equal(a[key], b[key]), key


def test_decode_config_both_schedules(moe):
    cfg = wl.CONFIGS["decode"]
    a = run_workload(moe, cfg, moe.MOE_SCHEDULE_AUTO)          # resolves to the fused decode schedule
    b = run_workload(moe, cfg, moe.MOE_SCHEDULE_PREFILL)
    for key in a:
        assert a[key].tobytes() == b[key].tobytes(), key        # schedules give identical values


@pytest.mark.parametrize("name", ["prefill", "skewed", "wide"])
def test_full_size_prefill_configs(moe, name):
    """Full benchmark sizes, in the launch configuration bench.py times, compared in full."""
    cfg = wl.CONFIGS[name]
    got = run_workload(moe, cfg, moe.MOE_SCHEDULE_AUTO)
    if name == "skewed":
        assert got["c_exp"].max() > 10 * cfg.N / cfg.E          # the hot experts really are hot


@pytest.mark.parametrize("T,H,k,E,R", [(19000, 7168, 2, 64, 8),      # X = 272 MB: two branches per dispatch unit
                                       (33000, 4096, 8, 128, 16)])   # X = 270 MB, one-wave slices: eight per unit
def test_batches_larger_than_the_infinity_cache(moe, T, H, k, E, R):
    """Token rows of more than 256 MiB: the prefill dispatch switches to larger units (it cannot find X cached)."""
    run_workload(moe, wl.Config("big-x", T=T, H=H, k=k, E=E, R=R, seed=T), moe.MOE_SCHEDULE_PREFILL)


# --------------------------------------------------------------------------- several tiles, ragged tails

@pytest.mark.parametrize("T,H,k,E,R", [
    (777, 7168, 8, 256, 32),     # 6216 branches: 7 plan tiles, ragged last tile and last wave round
    (1500, 4096, 6, 96, 12),     # E not a power of two, k not a power of two
    (333, 1032, 3, 1024, 64),    # E at the limit, rows of 129 vectors (ragged chunk)
    (2049, 512, 1, 4, 1),        # k = 1, one region
    (129, 8, 16, 16, 16),        # 16-byte rows, E = R
    (70001, 8, 8, 64, 8),        # 560008 branches: plan tiles of 2048 branches
    (140001, 8, 8, 64, 8),       # 1120008 branches: more than 512 tiles of 2048, so the tiles grow to 4096
])
@pytest.mark.parametrize("dtype", [wl.DTYPE_BF16, wl.DTYPE_F32])
def test_ragged_shapes(moe, T, H, k, E, R, dtype):
    if dtype == wl.DTYPE_F32:
        H = max(4, H // 2)
    cfg = wl.Config("ragged", T=T, H=H, k=k, E=E, R=R, dtype=dtype, seed=T)
    run_workload(moe, cfg, moe.MOE_SCHEDULE_PREFILL)


@pytest.mark.parametrize("T,H,k,E,R", [(1, 7168, 8, 256, 32), (37, 4096, 8, 128, 16), (255, 264, 8, 64, 8),
                                       (1024, 64, 8, 256, 32), (100, 2048, 20, 24, 3)])
def test_decode_schedule_matches_prefill(moe, T, H, k, E, R):
    cfg = wl.Config("dec", T=T, H=H, k=k, E=E, R=R, seed=T + 1)
    a = run_workload(moe, cfg, moe.MOE_SCHEDULE_DECODE)
    b = run_workload(moe, cfg, moe.MOE_SCHEDULE_PREFILL)
    for key in a:
        assert a[key].tobytes() == b[key].tobytes(), key


# --------------------------------------------------------------------------- degenerate routing

def _case(moe, K, E, R, schedule, H=64, stride=0, dtype=np.uint16, seed=0, label=""):
    rng = np.random.default_rng(seed)
    T, k = K.shape
    Xf = rng.standard_normal((T, H)).astype(np.float32)
    X = wl.f32_to_bf16_bits(Xf) if dtype == np.uint16 else Xf
    W = rng.random((T, k)).astype(np.float32)
    scale = rng.uniform(0.5, 1.5, E).astype(np.float32)
    return run_case(moe, X, K, W, scale, E, R, schedule, stride, label)


@pytest.mark.parametrize("schedule", ["prefill", "decode"])
def test_edge_cases(moe, schedule):
    sch = moe.MOE_SCHEDULE_PREFILL if schedule == "prefill" else moe.MOE_SCHEDULE_DECODE
    rng = np.random.default_rng(11)
    # no tokens
    _case(moe, np.zeros((0, 4), np.int32), 8, 2, sch, label="T=0")
    # one token, one slot
    _case(moe, np.array([[3]], np.int32), 8, 2, sch, label="T=1,k=1")
    # every branch to one expert (longest possible stream, maximal atomic contention)
    _case(moe, np.full((300, 4), 5, np.int32), 8, 4, sch, label="one expert")
    # duplicates inside a token and k > E
    _case(moe, wl.random_routing(rng, 90, 12, 5), 5, 5, sch, label="k>E duplicates")
    # masked slots and out-of-range ids
    _case(moe, wl.random_routing(rng, 200, 6, 32, p_masked=0.3, p_invalid=0.1), 32, 8, sch, label="masked+invalid")
    # everything masked
    _case(moe, np.full((17, 3), -1, np.int32), 4, 2, sch, label="all masked")
    # E = 1
    _case(moe, np.zeros((65, 2), np.int32), 1, 1, sch, label="E=1")
    # fp32 storage with masked slots
    _case(moe, wl.random_routing(rng, 70, 4, 16, p_masked=0.2), 16, 4, sch, H=36, dtype=np.float32, label="fp32")


@pytest.mark.parametrize("schedule", ["prefill", "decode"])
def test_fixed_stride_windows(moe, schedule):
    sch = moe.MOE_SCHEDULE_PREFILL if schedule == "prefill" else moe.MOE_SCHEDULE_DECODE
    rng = np.random.default_rng(12)
    K = wl.random_routing(rng, 250, 4, 16, distinct=True)
    tight = oracle.plan(K, 16, 4)
    roomy = int(tight.c_rank.max()) + 5
    got = _case(moe, K, 16, 4, sch, stride=roomy, label="stride roomy")
    assert got["status"][1] == 0
    tightest = int(np.sort(tight.c_rank)[1])            # some regions overflow
    got = _case(moe, K, 16, 4, sch, stride=tightest, label="stride overflow")
    assert got["status"][1] > 0 and (got["row_map"] == -1).sum() == got["status"][1]


def test_special_values_in_combine(moe):
    """Inf, NaN, signed zeros and subnormals travel through dispatch unchanged and through combine as in the oracle."""
    T, H, k, E, R = 8, 64, 2, 4, 2
    rng = np.random.default_rng(13)
    X = rng.integers(0, 2 ** 16, size=(T, H)).astype(np.uint16)         # arbitrary bf16 bit patterns
    X[0, :8] = [0x7F80, 0xFF80, 0x7FC0, 0x0000, 0x8000, 0x0001, 0x8001, 0x7F7F]
    K = wl.random_routing(rng, T, k, E, distinct=True)
    W = rng.standard_normal((T, k)).astype(np.float32)
    run_case(moe, X, K, W, np.ones(E, np.float32), E, R, moe.MOE_SCHEDULE_PREFILL, label="special values")


@pytest.mark.parametrize("T,H,k,E,R,dtype", [
    (4000, 4104, 6, 96, 12, np.uint16),      # k = 6; rows of 513 vectors: ragged last wave of every token
    (3100, 2056, 8, 64, 8, np.float32),      # fp32 storage, rows of 514 vectors
    (16001, 2048, 8, 32, 4, np.uint16),      # two rounds of the persistent grid with a ragged last round
])
def test_combine_streaming_form_with_masked_slots(moe, T, H, k, E, R, dtype):
    """Launches large enough for combine's deferred-store form (T * H * b / 16 above 1.5 Mi vectors, k of 6 or 8)
    with masked and out-of-range slots, on row lengths that are not a whole number of waves."""
    rng = np.random.default_rng(T)
    K = wl.random_routing(rng, T, k, E, distinct=True, p_masked=0.15, p_invalid=0.02)
    got = _case(moe, K, E, R, moe.MOE_SCHEDULE_PREFILL, H=H, dtype=dtype, seed=T, label="streaming combine")
    assert got["status"][0] > 0 and (got["row_map"] == -1).any()


def test_run_to_run_determinism(moe):
    cfg = wl.Config("det", T=3000, H=1024, k=8, E=256, R=32, routing="zipf", seed=5)
    a = run_workload(moe, cfg, moe.MOE_SCHEDULE_PREFILL)
    b = run_workload(moe, cfg, moe.MOE_SCHEDULE_PREFILL)
    for key in a:
        assert a[key].tobytes() == b[key].tobytes(), key


def test_identity_expert_round_trip_on_gpu(moe):
    """Dispatch then combine with the window itself as expert output and weights summing to 1
    restores the input to within 1 ulp (the spec invariant), here on the GPU path alone."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    cfg = wl.CONFIGS["decode"]
    w = wl.make(cfg)
    layer = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, separate_expert_out=False)
    layer.dispatch(to_device(w.X), to_device(w.K))
    layer.combine(to_device(w.W))
    torch.cuda.synchronize()
    assert max_ulp(to_host(layer.y), w.X) <= 1
    # the pre-marshalled calls do the same thing
    first = to_host(layer.y).copy()
    layer.y.zero_(), layer.window.zero_()
    dispatch, combine = layer.bind(to_device(w.X), to_device(w.K), to_device(w.W))
    dispatch()
    combine()
    torch.cuda.synchronize()
    assert to_host(layer.y).tobytes() == first.tobytes()


def test_hip_graph_replay_matches_eager(moe):
    """A captured dispatch -> combine pair (kernel nodes only) replayed several times, with eager work
    and synchronisations in between, gives the eager result on every replay -- also after the inputs
    were overwritten in place with a different batch."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    cfg = wl.CONFIGS["decode"].with_(T=96, H=2048)
    layer = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, separate_expert_out=False)
    eager = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, separate_expert_out=False)
    w0 = wl.make(cfg, seed=21)
    xd, kd, wd = to_device(w0.X), to_device(w0.K), to_device(w0.W)
    layer.dispatch(xd, kd)                  # warm-up outside the capture
    layer.combine(wd)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        layer.dispatch(xd, kd)
        layer.combine(wd)
    for rep in range(5):
        w = wl.make(cfg, seed=30 + rep)
        xd.copy_(to_device(w.X)), kd.copy_(to_device(w.K)), wd.copy_(to_device(w.W))
        layer.window.zero_(), layer.y.zero_(), layer.plan.row_map.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        eager.dispatch(xd, kd)
        eager.combine(wd)
        torch.cuda.synchronize()
        ref = oracle.plan(w.K, cfg.E, cfg.R)
        assert np.array_equal(to_host(layer.plan.row_map).reshape(cfg.T, cfg.k), ref.row_map), rep
        assert to_host(layer.window).tobytes() == to_host(eager.window).tobytes(), rep
        assert to_host(layer.y).tobytes() == to_host(eager.y).tobytes(), rep
        assert to_host(layer.window).tobytes() == oracle.dispatch(w.X, ref.row_map, ref.window_rows).tobytes(), rep


def test_hip_graph_replay_of_a_prefill_layer(moe):
    """plan -> dispatch -> combine of a streaming-size layer (two-launch plan, sliced dispatch, deferred-store
    combine) captured once and replayed on changing inputs: every replay equals the eager result and the oracle."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    cfg = wl.CONFIGS["prefill"].with_(T=4096, H=4096, E=64, R=8)
    layer = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, schedule=moe.MOE_SCHEDULE_PREFILL, separate_expert_out=False)
    eager = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, schedule=moe.MOE_SCHEDULE_PREFILL, separate_expert_out=False)
    w0 = wl.make(cfg, seed=41)
    xd, kd, wd = to_device(w0.X), to_device(w0.K), to_device(w0.W)

    def run(l):
        moe.moe_plan(l.shape, kd, l.plan)
        l.dispatch(xd, kd)
        l.combine(wd)

    run(layer)                              # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(layer)
    for rep in range(3):
        w = wl.make(cfg, seed=50 + rep)
        xd.copy_(to_device(w.X)), kd.copy_(to_device(w.K)), wd.copy_(to_device(w.W))
        layer.window.zero_(), layer.y.zero_(), layer.plan.row_map.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        run(eager)
        torch.cuda.synchronize()
        ref = oracle.plan(w.K, cfg.E, cfg.R)
        print(f"[graph prefill] replay {rep}", flush=True)
        assert np.array_equal(to_host(layer.plan.row_map).reshape(cfg.T, cfg.k), ref.row_map), rep
        assert to_host(layer.window).tobytes() == oracle.dispatch(w.X, ref.row_map, ref.window_rows).tobytes(), rep
        assert to_host(layer.y).tobytes() == to_host(eager.y).tobytes(), rep
        assert max_ulp(to_host(layer.y), w.X) <= 1, rep        # identity expert, weights sum to 1


# --------------------------------------------------------------------------- several source ranks (Notify with M)

def run_multi(moe, cfg, M, me, schedule, stride=0, seed=0):
    """Plan / dispatch / combine of source rank `me` next to the blocks of the other sources."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    w = wl.make(cfg, seed=seed)
    T, k, E, R = cfg.T, cfg.k, cfg.E, cfg.R
    ref = oracle.plan_multi(w.K, M, me, E, R, stride)
    rows = max(1, R * stride if stride else ref.window_rows)
    print(f"[multi] T={T} E={E} R={R} me={me} schedule={schedule} stride={stride} rows={rows}", flush=True)
    layer = MoeLayer(T, cfg.H, k, E, R, schedule=schedule, region_stride_rows=stride, rank_id=me,
                     source_count=to_device(M), window_rows=rows)
    fill = SENTINEL[np.dtype(np.uint16)]
    layer.window.copy_(to_device(np.full(tuple(layer.window.shape), fill, np.uint16)))
    xd = to_device(w.X) if T else torch.empty((1, cfg.H), dtype=torch.bfloat16, device="cuda")
    kd = to_device(w.K) if T else torch.empty((1, k), dtype=torch.int32, device="cuda")
    wd = to_device(w.W) if T else torch.empty((1, k), dtype=torch.float32, device="cuda")
    if layer.schedule == moe.MOE_SCHEDULE_PREFILL:
        moe.moe_plan(layer.shape, kd, layer.plan)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(layer.plan.row_map)[:T * k].reshape(T, k), ref.row_map), "row_map (plan only)"
    layer.dispatch(xd, kd)
    torch.cuda.synchronize()
    p = layer.plan
    assert np.array_equal(to_host(p.expert_count), ref.c_exp)
    assert np.array_equal(to_host(p.rank_count), ref.c_rank)
    assert np.array_equal(to_host(p.expert_offset), ref.expert_offset)
    assert np.array_equal(to_host(p.region_base), ref.region_base)
    assert np.array_equal(to_host(p.recv_count), ref.recv_count)
    assert np.array_equal(to_host(p.recv_offset), ref.recv_offset)
    assert np.array_equal(to_host(p.send_idx)[:T * k].reshape(T, k), ref.s)
    assert np.array_equal(to_host(p.row_map)[:T * k].reshape(T, k), ref.row_map)
    assert np.array_equal(to_host(p.status)[:3], ref.status)
    ref_window = oracle.dispatch(w.X, ref.row_map, rows, fill=fill)        # other sources' rows stay untouched
    assert to_host(layer.window)[:rows].tobytes() == ref_window.tobytes()
    Yexp = oracle.expert_standin(ref_window, w.K, ref.row_map, w.scale)
    layer.expert_out[:rows].copy_(to_device(Yexp))
    layer.combine(wd)
    torch.cuda.synchronize()
    assert max_ulp(to_host(layer.y)[:T], oracle.combine(Yexp, w.W, ref.row_map)) <= 1
    return ref


@pytest.mark.parametrize("schedule", ["prefill", "decode"])
def test_multi_source_notify(moe, schedule):
    sch = moe.MOE_SCHEDULE_PREFILL if schedule == "prefill" else moe.MOE_SCHEDULE_DECODE
    rng = np.random.default_rng(40)
    for (T, H, k, E, R) in ((200, 256, 8, 64, 8), (77, 64, 4, 12, 4), (1000, 128, 8, 256, 32), (5, 64, 2, 8, 1)):
        cfg = wl.Config("multi", T=T, H=H, k=k, E=E, R=R, seed=T)
        M = rng.integers(0, 40, size=(R, E)).astype(np.int32)
        for me in sorted({0, R // 2, R - 1}):
            ref = run_multi(moe, cfg, M, me, sch, seed=T + me)
            assert ref.window_rows > T * k or R == 1
        # fixed stride, some regions overflowing
        full = M.copy()
        per_region = full.reshape(R, R, E // R).sum(axis=(0, 2)) + T * k // R
        stride = int(np.sort(per_region)[R // 2])
        ref = run_multi(moe, cfg, M, R - 1, sch, stride=stride, seed=T)
    # no tokens on this rank, but other sources present
    cfg = wl.Config("multi0", T=0, H=64, k=4, E=16, R=4)
    run_multi(moe, cfg, rng.integers(0, 9, size=(4, 16)).astype(np.int32), 2, sch)
    # zero matrix == single source
    cfg = wl.Config("multiz", T=300, H=64, k=8, E=32, R=4, seed=9)
    ref = run_multi(moe, cfg, np.zeros((4, 32), np.int32), 3, sch, seed=9)
    assert np.array_equal(ref.expert_offset, oracle.plan(wl.make(cfg, seed=9).K, 32, 4).expert_offset)


def test_plan_on_both_sides_of_the_single_launch_limit(moe):
    """The explicit plan runs as one launch up to 12 tiles of 1024 branches and as two launches above:
    the same cases (masked and invalid ids, fixed stride, several source ranks, skewed routing) on both sides."""
    rng = np.random.default_rng(77)
    for T in (1535, 1536, 1537, 2500):                # N = 12280, 12288 (last single launch), 12296, 20000
        cfg = wl.CONFIGS["skewed"].with_(T=T, H=64, E=64, R=8)
        w = wl.make(cfg, seed=T)
        K = w.K.copy()
        K[rng.integers(0, T, 40), rng.integers(0, cfg.k, 40)] = -1
        K[rng.integers(0, T, 9), rng.integers(0, cfg.k, 9)] = cfg.E + 3
        run_case(moe, w.X, K, w.W, w.scale, cfg.E, cfg.R, moe.MOE_SCHEDULE_PREFILL, label=f"limit T={T}")
        run_case(moe, w.X, K, w.W, w.scale, cfg.E, cfg.R, moe.MOE_SCHEDULE_PREFILL, stride=T * cfg.k // cfg.R,
                 label=f"limit T={T} fixed stride")
        M = rng.integers(0, 300, size=(cfg.R, cfg.E)).astype(np.int32)
        run_multi(moe, cfg, M, cfg.R // 2, moe.MOE_SCHEDULE_PREFILL, seed=T)


# --------------------------------------------------------------------------- row-wise quantised dispatch

def run_quant(moe, cfg, schedule, stride=0, seed=0, scale_rows=None, plant=None):
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    w = wl.make(cfg, seed=seed)
    X = w.X.copy()
    if scale_rows is not None:                       # per-row magnitudes spread over many binades
        f = wl.bf16_bits_to_f32(X) * scale_rows[:, None]
        X = wl.f32_to_bf16_bits(f.astype(np.float32))
    if plant is not None:                            # (row, column, bf16 bits) triples: Inf / NaN elements
        for (r, c, bits) in plant:
            X[r, c] = bits
    T, H, k, E, R = cfg.T, cfg.H, cfg.k, cfg.E, cfg.R
    ref = oracle.plan(w.K, E, R, stride)
    layer = MoeLayer(T, H, k, E, R, schedule=schedule, region_stride_rows=stride)
    rows = layer.rows
    print(f"[quant] T={T} H={H} k={k} E={E} schedule={schedule} stride={stride}", flush=True)
    wq = torch.full((max(rows, 1), H), 0xAA, dtype=torch.uint8, device="cuda")
    ws = torch.full((max(rows, 1),), -1.0, dtype=torch.float32, device="cuda")
    xd, kd = to_device(X), to_device(w.K)
    if layer.schedule == moe.MOE_SCHEDULE_PREFILL:
        moe.moe_plan(layer.shape, kd, layer.plan)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(layer.plan.row_map)[:T * k].reshape(T, k), ref.row_map)
    moe.moe_dispatch_quant(layer.shape, xd, kd, layer.plan, wq, ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(layer.plan.row_map)[:T * k].reshape(T, k), ref.row_map)
    assert np.array_equal(to_host(layer.plan.expert_count), ref.c_exp)
    ref_q, ref_s = oracle.dispatch_quant(X, ref.row_map, max(rows, 1), fill=0xAA)
    got_q, got_s = wq.cpu().numpy(), ws.cpu().numpy()
    assert got_s.tobytes() == ref_s.tobytes(), "row scales"
    # a NaN code is S.1111.111 with either sign: which sign a NaN product carries is not part of the format
    both_nan = ((got_q & 0x7F) == 0x7F) & ((ref_q & 0x7F) == 0x7F)
    bad = np.count_nonzero((got_q != ref_q) & ~both_nan)
    assert bad == 0, f"{bad} of {got_q.size} fp8 codes differ"
    return got_q, got_s


@pytest.mark.parametrize("schedule", ["prefill", "decode"])
def test_quantised_dispatch(moe, schedule):
    sch = moe.MOE_SCHEDULE_PREFILL if schedule == "prefill" else moe.MOE_SCHEDULE_DECODE
    rng = np.random.default_rng(50)
    for (T, H, k, E, R) in ((128, 7168, 8, 256, 32), (100, 4096, 8, 128, 16), (61, 1032, 3, 12, 4), (200, 64, 8, 32, 4),
                            (9, 16384, 4, 8, 2), (33, 30000 // 8 * 8, 2, 4, 1)):
        cfg = wl.Config("quant", T=T, H=H, k=k, E=E, R=R, seed=T)
        run_quant(moe, cfg, sch, seed=T, scale_rows=np.exp(rng.uniform(-8, 8, T)).astype(np.float32))
    cfg = wl.Config("quant", T=64, H=512, k=4, E=16, R=4, seed=3)
    zero = np.ones(64, np.float32)
    zero[::5] = 0.0                                   # all-zero rows: scale 1, codes 0
    run_quant(moe, cfg, sch, seed=3, scale_rows=zero)
    run_quant(moe, cfg, sch, stride=70, seed=4)       # fixed stride with overflow
    # non-finite inputs: a NaN element gives a NaN code and does not enter amax; a row with an infinite
    # element has scale +Inf, zero codes (signed) for its finite elements and NaN codes for the infinite ones
    PINF, NINF, NAN, NNAN = 0x7F80, 0xFF80, 0x7FC0, 0xFFC1
    q, sc = run_quant(moe, cfg, sch, seed=5, plant=[(0, 3, NAN), (0, 100, NNAN), (1, 7, PINF), (2, 9, NINF),
                                                    (2, 10, NAN), (3, 0, PINF), (3, 511, NINF)])
    assert np.isinf(sc).sum() >= 1 and not np.isnan(sc).any()


@pytest.mark.parametrize("schedule", ["prefill", "decode"])
def test_quantised_dispatch_with_several_sources(moe, schedule):
    """Quantised rows land in the sub-blocks the several-sources plan assigns; the other sources' rows and scales
    stay untouched."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    sch = moe.MOE_SCHEDULE_PREFILL if schedule == "prefill" else moe.MOE_SCHEDULE_DECODE
    rng = np.random.default_rng(60)
    for (T, H, k, E, R) in ((128, 7168, 8, 256, 32), (300, 1024, 8, 64, 8), (50, 520, 3, 12, 4)):
        cfg = wl.Config("quant-multi", T=T, H=H, k=k, E=E, R=R, seed=T)
        w = wl.make(cfg)
        M = rng.integers(0, 30, size=(R, E)).astype(np.int32)
        me = R // 2
        ref = oracle.plan_multi(w.K, M, me, E, R)
        rows = ref.window_rows
        print(f"[quant multi] T={T} H={H} k={k} E={E} R={R} schedule={schedule} rows={rows}", flush=True)
        layer = MoeLayer(T, H, k, E, R, schedule=sch, rank_id=me, source_count=to_device(M), window_rows=rows)
        wq = torch.full((rows, H), 0xAA, dtype=torch.uint8, device="cuda")
        ws = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda")
        xd, kd = to_device(w.X), to_device(w.K)
        if sch == moe.MOE_SCHEDULE_PREFILL:
            moe.moe_plan(layer.shape, kd, layer.plan)
        moe.moe_dispatch_quant(layer.shape, xd, kd, layer.plan, wq, ws)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(layer.plan.row_map)[:T * k].reshape(T, k), ref.row_map)
        assert np.array_equal(to_host(layer.plan.recv_offset), ref.recv_offset)
        ref_q, ref_s = oracle.dispatch_quant(w.X, ref.row_map, rows, fill=0xAA)
        assert ws.cpu().numpy().tobytes() == ref_s.tobytes(), "row scales"
        assert wq.cpu().numpy().tobytes() == ref_q.tobytes(), "fp8 codes"
        assert (ref_s == -1.0).sum() == rows - T * k          # the other sources' rows were left alone


def test_quantised_dispatch_full_prefill(moe):
    run_quant(moe, wl.CONFIGS["prefill"], moe.MOE_SCHEDULE_AUTO)


# --------------------------------------------------------------------------- seeded shape fuzz

def test_seeded_random_shapes(moe):
    """Forty seeded shapes over both schedules: odd sizes, masked / invalid / duplicate ids, fixed strides,
    several source ranks, fp32 and bf16 storage, routing degrees up to 100 and E up to the limit.
    MOE_FUZZ_CASES / MOE_FUZZ_SEED in the environment run a longer or a different series."""
    rng = np.random.default_rng(int(os.environ.get("MOE_FUZZ_SEED", "2024")))
    from paper_2605_06055_amd.layer import to_device
    for case in range(int(os.environ.get("MOE_FUZZ_CASES", "40"))):
        R = int(rng.choice([1, 2, 3, 4, 8, 16, 32]))
        Er = int(rng.choice([1, 2, 3, 8, 32]))
        E = min(R * Er, 1024)
        R = E // Er
        k = int(rng.choice([1, 2, 3, 8, 9, 16, 64, 100]))
        decode = bool(rng.integers(0, 2))
        T = int(rng.integers(1, max(2, 8192 // k))) if decode else int(rng.integers(1, 3000))
        if decode and T * k > 8192:
            T = 8192 // k
        dtype = np.uint16 if rng.random() < 0.7 else np.float32
        H = int(rng.integers(1, 300)) * (8 if dtype == np.uint16 else 4)
        K = wl.random_routing(rng, T, k, E, distinct=bool(rng.integers(0, 2)), p_masked=float(rng.choice([0, 0.1])),
                              p_invalid=float(rng.choice([0, 0.05])))
        sch = moe.MOE_SCHEDULE_DECODE if decode else moe.MOE_SCHEDULE_PREFILL
        tight = oracle.plan(K, E, R)
        stride = 0
        if rng.random() < 0.3:
            stride = max(1, int(tight.c_rank.max() * rng.uniform(0.6, 1.3)))
        _case(moe, K, E, R, sch, H=H, stride=stride, dtype=dtype, seed=case, label=f"fuzz {case}")


def test_seeded_large_shapes(moe):
    """Seeded shapes of the size where the prefill path changes form: two-launch plan, order list on and off,
    deferred-store combine, with masked / invalid ids and sometimes a fixed stride.  MOE_FUZZ_LARGE_CASES /
    MOE_FUZZ_SEED run a longer or a different series."""
    rng = np.random.default_rng(int(os.environ.get("MOE_FUZZ_SEED", "2025")) + 1)
    for case in range(int(os.environ.get("MOE_FUZZ_LARGE_CASES", "5"))):
        H = int(rng.choice([1024, 1544, 2048, 4096, 5128, 6144, 7168, 8192]))
        k = int(rng.choice([4, 6, 8]))
        R = int(rng.choice([4, 8, 32]))
        E = R * int(rng.choice([2, 8]))
        T = int(rng.integers(1600, 7000))
        K = wl.random_routing(rng, T, k, E, distinct=True, p_masked=float(rng.choice([0, 0.05])),
                              p_invalid=float(rng.choice([0, 0.01])))
        stride = 0
        if rng.random() < 0.25:
            stride = max(1, int(oracle.plan(K, E, R).c_rank.max() * rng.uniform(0.8, 1.2)))
        _case(moe, K, E, R, moe.MOE_SCHEDULE_PREFILL, H=H, stride=stride, seed=case, label=f"large fuzz {case}")


def check_order_list(order, K, ref, E):
    """The plan's dispatch order list: every counted branch once as (token, window row), unused entries (-1, -1),
    rows non-decreasing inside every aligned run of 1024 entries (a piece of one sorted stretch)."""
    T, k = K.shape
    N = T * k
    pairs = order[:2 * N].reshape(N, 2)
    flat = K.reshape(-1)
    counted = (flat >= 0) & (flat < E)
    want = np.stack([np.repeat(np.arange(T), k)[counted], ref.row_map.reshape(-1)[counted]], axis=1)
    used = pairs[:, 0] >= 0
    assert used.sum() == counted.sum()
    assert np.all(pairs[~used] == -1)
    key = lambda a: a[np.lexsort((a[:, 0], a[:, 1]))]
    placed_got, placed_want = pairs[used & (pairs[:, 1] >= 0)], want[want[:, 1] >= 0]
    assert np.array_equal(key(placed_got), key(placed_want))                  # rows are unique: pairs match one to one
    assert np.array_equal(np.sort(pairs[used & (pairs[:, 1] < 0)][:, 0]), np.sort(want[want[:, 1] < 0][:, 0]))
    for a in range(0, N, 1024):
        rows = pairs[a:a + 1024, 1]
        rows = rows[rows >= 0]
        assert np.all(np.diff(rows) >= 0), f"list entries {a}.. are not sorted by window row"


def test_dispatch_order_list(moe):
    """Where the shape qualifies (rows of at least 12 KB: X up to 96 MiB and windows up to 770 MiB; rows of 8 to
    12 KB and of 2 to 4 KB: windows up to 1100 MiB) the plan also emits the placed
    branches sorted by window row inside stretches of tokens, and dispatch walks that list.  The list is checked
    against the oracle's row map, and dispatch must give the same window with and without it."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    rng = np.random.default_rng(91)
    cases = [(777, 7168, 8, 256, 32, 0, False),       # one launch plan: the batch is one stretch
             (6000, 4096, 8, 64, 8, 0, False),        # two launches, two units per workgroup, two stretches of 24 tiles
             (2900, 7168, 8, 256, 32, 0, False),      # two stretches of 12 tiles, ragged last one
             (7000, 7168, 8, 256, 32, 0, False),      # just under the limit on X (96 MiB): four stretches of 14 tiles
             (2600, 4096, 8, 64, 8, 2000, False),     # fixed stride with dropped branches
             (2100, 8200, 6, 48, 4, 0, True),         # several source ranks, ragged row tail
             (1300, 2048, 9, 40, 5, 0, False),        # fp32 storage below (rows of 8 KB)
             (5000, 2040, 8, 64, 8, 0, False),        # rows of 255 vectors: four units of 32 lanes per workgroup
             (3000, 1024, 8, 32, 4, 0, False),        # rows of 2 KB: eight units of 16 lanes per workgroup
             (2000, 1544, 6, 48, 4, 900, True)]       # rows of 193 vectors (ragged slices), fixed stride, several sources
    for (T, H, k, E, R, stride, multi) in cases:
        fp32 = H == 2048
        K = wl.random_routing(rng, T, k, E, distinct=k <= E, p_masked=0.03, p_invalid=0.01)
        Xf = rng.standard_normal((T, H)).astype(np.float32)
        X = Xf if fp32 else wl.f32_to_bf16_bits(Xf)
        M = rng.integers(0, 50, size=(R, E)).astype(np.int32) if multi else None
        me = R // 2
        ref = oracle.plan_multi(K, M, me, E, R, stride) if multi else oracle.plan(K, E, R, stride)
        rows = R * stride if stride else max(ref.window_rows, T * k)      # the caller provides moe_window_rows rows
        windows = []
        for with_order in (True, False):
            print(f"[order] T={T} H={H} k={k} E={E} stride={stride} multi={multi} list={with_order}", flush=True)
            layer = MoeLayer(T, H, k, E, R, dtype=moe.MOE_DTYPE_F32 if fp32 else moe.MOE_DTYPE_BF16,
                             schedule=moe.MOE_SCHEDULE_PREFILL, region_stride_rows=stride, rank_id=me if multi else 0,
                             source_count=None if M is None else to_device(M), window_rows=rows)
            if not with_order:
                layer.plan.dispatch_order = None
                layer._plan_struct = layer.plan.struct()
            else:
                layer.plan.dispatch_order.fill_(-77)
            layer.window.view(torch.int16).fill_(0x7B7B)
            layer.dispatch(to_device(X), to_device(K))
            torch.cuda.synchronize()
            assert np.array_equal(to_host(layer.plan.row_map)[:T * k].reshape(T, k), ref.row_map)
            if with_order:
                check_order_list(to_host(layer.plan.dispatch_order), K, ref, E)
            windows.append(to_host(layer.window.view(torch.int16))[:rows])
        assert windows[0].tobytes() == windows[1].tobytes()
        fill = np.uint16(0x7B7B) if not fp32 else np.frombuffer(np.array([0x7B7B, 0x7B7B], np.uint16).tobytes(), np.float32)[0]
        want = oracle.dispatch(X, ref.row_map, rows, fill=fill)
        assert windows[0].tobytes() == want.tobytes()


def test_plan_prefetch_changes_nothing(moe):
    """moe_plan_t.prefetch only makes spare workgroups of the plan read a range of memory: every plan output is
    what it is without it, for the one-launch and the two-launch plan, for moe_plan_static, for ranges that are
    not a whole number of workgroup chunks and for ranges beyond what the plan reads at most."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    for (T, H, k, E, R) in ((1000, 1032, 8, 64, 8), (4096, 2048, 8, 256, 32), (3000, 7168, 8, 256, 32)):
        cfg = wl.Config("prefetch", T=T, H=H, k=k, E=E, R=R, seed=T)
        w = wl.make(cfg)
        ref = oracle.plan(w.K, E, R)
        xd, kd = to_device(w.X), to_device(w.K)
        big = torch.zeros((225 << 20) // 4 + 4, dtype=torch.int32, device="cuda")       # more than the plan reads
        for call in (moe.moe_plan, moe.moe_plan_static):
            for what in (xd, xd.view(-1)[:T * H - 8 * 37], big):
                layer = MoeLayer(T, H, k, E, R, schedule=moe.MOE_SCHEDULE_PREFILL)
                layer.plan.prefetch = what
                for t in (layer.plan.row_map, layer.plan.send_idx, layer.plan.expert_offset):
                    t.fill_(-9)
                print(f"[prefetch] T={T} H={H} {call.__name__} bytes={what.numel() * what.element_size()}", flush=True)
                call(layer.shape, kd, layer.plan)
                torch.cuda.synchronize()
                assert np.array_equal(to_host(layer.plan.row_map)[:T * k].reshape(T, k), ref.row_map)
                assert np.array_equal(to_host(layer.plan.send_idx)[:T * k].reshape(T, k), ref.s)
                assert np.array_equal(to_host(layer.plan.expert_offset), ref.expert_offset)
                assert np.array_equal(to_host(layer.plan.status)[:3], ref.status)
        # a whole layer through MoeLayer with the hint switched on
        layer = MoeLayer(T, H, k, E, R, schedule=moe.MOE_SCHEDULE_PREFILL)
        layer.prefetch_x = True
        layer.dispatch(xd, kd)
        torch.cuda.synchronize()
        assert to_host(layer.window).tobytes() == oracle.dispatch(w.X, ref.row_map, ref.window_rows).tobytes()


def test_plan_left_by_decode_dispatch_is_reusable(moe):
    """A later call on identical routing may skip planning: the explicit schedule's dispatch, given the plan
    state a fused decode dispatch left behind, places new payload in the same rows."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    from paper_2605_06055_amd import binding as B
    cfg = wl.CONFIGS["decode"]
    w = wl.make(cfg)
    ref = oracle.plan(w.K, cfg.E, cfg.R)
    layer = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, schedule=moe.MOE_SCHEDULE_DECODE)
    kd = to_device(w.K)
    layer.dispatch(to_device(w.X), kd)                               # plans and places X
    X2 = wl.make(cfg, seed=99).X                                     # new payload, same routing
    reuse = B.MoeShape(T=cfg.T, H=cfg.H, k=cfg.k, E=cfg.E, R=cfg.R, dtype=moe.MOE_DTYPE_BF16,
                       schedule=moe.MOE_SCHEDULE_PREFILL, rank_id=0, region_stride_rows=0)
    moe.moe_dispatch(reuse, to_device(X2), None, layer.plan, layer.window)      # no moe_plan, no ids
    torch.cuda.synchronize()
    assert np.array_equal(to_host(layer.plan.row_map).reshape(cfg.T, cfg.k), ref.row_map)
    assert to_host(layer.window).tobytes() == oracle.dispatch(X2, ref.row_map, ref.window_rows).tobytes()


@pytest.mark.parametrize("T,H,k", [(112, 4104, 8), (128, 8200, 8), (300, 8192, 3), (1024, 16392, 8), (100, 4104, 9)])
def test_decode_dispatch_wide_rows(moe, T, H, k):
    """Rows wider than one workgroup pass (more than 512 16-byte columns) on both sides of the batch size at
    which the fused dispatch switches to two vectors per lane (896 branches), with ragged row tails, masked
    and invalid ids, a fixed stride and several source ranks."""
    rng = np.random.default_rng(T + H)
    E, R = 64, 8
    K = wl.random_routing(rng, T, k, E, distinct=True, p_masked=0.05, p_invalid=0.02)
    a = _case(moe, K, E, R, moe.MOE_SCHEDULE_DECODE, H=H, seed=T, label=f"wide rows T={T} H={H}")
    b = _case(moe, K, E, R, moe.MOE_SCHEDULE_PREFILL, H=H, seed=T, label=f"wide rows T={T} H={H} (explicit)")
    for key in a:
        assert np.array_equal(a[key], b[key]), key
    _case(moe, K, E, R, moe.MOE_SCHEDULE_DECODE, H=H, stride=max(1, T * k // R), seed=T, label="wide rows, fixed stride")
    cfg = wl.Config("widerows", T=T, H=H, k=k, E=E, R=R, seed=T)
    run_multi(moe, cfg, rng.integers(0, 50, size=(R, E)).astype(np.int32), R // 2, moe.MOE_SCHEDULE_DECODE, seed=T)


def test_decode_schedule_limits(moe):
    """Largest batch the fused decode kernel accepts (8192 branches) with the largest expert count."""
    rng = np.random.default_rng(77)
    K = wl.random_routing(rng, 1024, 8, 1024, distinct=True)
    _case(moe, K, 1024, 128, moe.MOE_SCHEDULE_DECODE, H=64, label="decode N=8192 E=1024")
    K = wl.random_routing(rng, 64, 128, 1024)          # k = 128 with duplicates
    _case(moe, K, 1024, 1024, moe.MOE_SCHEDULE_DECODE, H=8, label="decode k=128 E=R=1024")


def test_optional_outputs_and_side_stream(moe):
    """send_idx / recv tables may be NULL; calls issued on a non-default stream stay on that stream."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    from paper_2605_06055_amd.binding import _PlanStruct
    for cfg, sch in ((wl.Config("opt", T=700, H=256, k=8, E=64, R=8, seed=1), moe.MOE_SCHEDULE_PREFILL),
                     (wl.Config("opt", T=90, H=256, k=8, E=64, R=8, seed=2), moe.MOE_SCHEDULE_DECODE)):
        w = wl.make(cfg)
        ref_plan, ref_window, ref_yexp, ref_y = oracle.layer(w.X, w.K, w.W, w.scale, cfg.E, cfg.R)
        layer = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, schedule=sch)
        p = layer.plan
        p.workspace.fill_(0x5A)                                   # stale scratch must not matter
        ps = _PlanStruct(p.expert_count.data_ptr(), p.rank_count.data_ptr(), p.expert_offset.data_ptr(),
                         p.region_base.data_ptr(), None, p.row_map.data_ptr(), p.status.data_ptr(),
                         p.workspace.data_ptr(), p.workspace.numel(), None, None, None)
        p.send_idx.fill_(-9)
        side = torch.cuda.Stream()
        xd, kd, wd = to_device(w.X), to_device(w.K), to_device(w.W)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            if sch == moe.MOE_SCHEDULE_PREFILL:
                moe.moe_plan(layer.shape, kd, ps)
            moe.moe_dispatch(layer.shape, xd, kd, ps, layer.window)
            layer.expert_out.copy_(to_device(ref_yexp))
            moe.moe_combine(layer.shape, layer.expert_out, wd, ps, layer.y)
        side.synchronize()
        assert np.all(to_host(p.send_idx) == -9)                  # not written when NULL was passed
        assert np.array_equal(to_host(p.row_map).reshape(cfg.T, cfg.k), ref_plan.row_map)
        assert to_host(layer.window).tobytes() == ref_window.tobytes()
        assert max_ulp(to_host(layer.y), ref_y) <= 1


def test_two_layers_on_two_streams_concurrently(moe):
    """The library keeps no state between calls: two layers issued on two streams at the same time
    (prefill schedule on one, fused decode schedule on the other) both match the oracle."""
    from paper_2605_06055_amd.layer import MoeLayer, to_device, to_host
    jobs = []
    for cfg, sch in ((wl.Config("a", T=3000, H=2048, k=8, E=256, R=32, seed=61), moe.MOE_SCHEDULE_PREFILL),
                     (wl.Config("b", T=120, H=7168, k=8, E=256, R=32, seed=62), moe.MOE_SCHEDULE_DECODE)):
        w = wl.make(cfg)
        ref = oracle.layer(w.X, w.K, w.W, w.scale, cfg.E, cfg.R)
        layer = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, schedule=sch)
        layer.expert_out.copy_(to_device(ref[2]))
        jobs.append((layer, to_device(w.X), to_device(w.K), to_device(w.W), ref, torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(10):
        for layer, xd, kd, wd, ref, st in jobs:
            with torch.cuda.stream(st):
                layer.dispatch(xd, kd)
                layer.combine(wd)
    torch.cuda.synchronize()
    for layer, xd, kd, wd, ref, st in jobs:
        assert np.array_equal(to_host(layer.plan.row_map).reshape(ref[0].row_map.shape), ref[0].row_map)
        assert to_host(layer.window).tobytes() == ref[1].tobytes()
        assert max_ulp(to_host(layer.y), ref[3]) <= 1


def test_c_abi_from_a_plain_host_program(moe):
    """tests/abi_check (built by __graft_entry__.build) drives the library from C++ with hipMalloc'd
    buffers and its own stream, without Python or torch in the process, and checks against the oracle."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_check")
    if not os.path.exists(exe):
        pytest.skip("tests/abi_check has not been built (run __graft_entry__.build())")
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(res.stdout, res.stderr, flush=True)
    assert res.returncode == 0 and "abi_check: ok" in res.stdout
