#!/usr/bin/env python3
"""Benchmark of the relay-buffer-free MoE dispatch + combine path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch:
    prefill schedule : moe_plan -> moe_dispatch -> moe_combine   (3 calls, 4 kernels)
    decode schedule  : moe_dispatch (plan fused) -> moe_combine  (2 calls, 2 kernels)
with all inputs resident in HBM.  The stand-in expert that fills expert_out runs once, untimed.
`value` = algorithmic payload bytes of one step, 2*T*H*b*(1+k), divided by the step time.
Every step of a prefill workload reads the same X, so the Infinity Cache may still hold it from the step
before (as it holds a tensor that the preceding operator has just written); `x_cold` reports the headline
layer with X rotating through 8 copies, without and with the plan's prefetch hint.

Prints ONE JSON line on stdout (headline workload); details go to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E published peak
DESCR = {
    "prefill": "prefill balanced: T=4096 H=7168 bf16, E=256 in R=32 regions, top-8 uniform",
    "decode": "decode: T=128 H=7168 bf16, E=256 in R=32 regions, top-8 uniform",
    "skewed": "prefill skewed: T=16384 H=7168 bf16, E=256 in R=32 regions, top-8 Zipf(1.2)",
    "wide": "prefill wide: T=32768 H=4096 bf16, E=128 in R=16 regions, group-limited top-8",
}


def rounded(kern):
    return {k: (round(v, 2) if isinstance(v, float) else v) for k, v in kern.items()}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def event_percentiles_us(fn, iters, per_call=1):
    """p10/p50/p90 of the duration of single fn() calls (microseconds, divided by per_call), each
    bracketed by its own pair of HIP events; the calls still run back to back."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(ev):
        a.record()
        fn(i)
        b.record()
    torch.cuda.synchronize()
    d = sorted(a.elapsed_time(b) * 1e3 / per_call for a, b in ev)
    pick = lambda q: round(d[min(len(d) - 1, int(q * len(d)))], 2)
    return {"p10": pick(0.10), "p50": pick(0.50), "p90": pick(0.90), "samples": len(d)}


def event_time_ms(fn, iters):
    """Average duration of fn() over `iters` back-to-back calls, HIP events on the launch stream."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(iters):
        fn(i)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


class Sets:
    """`n` disjoint buffer sets of one workload (rotating through them keeps small working sets
    out of the 256 MB Infinity Cache between steps)."""

    def __init__(self, cfg, n, schedule=0, sources=1, quant=False):
        import torch
        import numpy as np
        import workloads as wl
        import paper_2605_06055_amd as moe
        from paper_2605_06055_amd.layer import MoeLayer, to_device
        from workloads.standin import standin_expert
        self.cfg, self.n, self.moe = cfg, n, moe
        self.layers, self.x, self.k, self.w = [], [], [], []
        self.quant, self.wq, self.ws = quant, [], []
        for i in range(n):
            w = wl.make(cfg, seed=cfg.seed + i)
            extra = {}
            if sources > 1:
                # the other source ranks route like this one: their counts are draws of the same routing law
                # (this rank is source rank R/2; rows of the other sources are never touched here)
                M = wl.source_count_matrix(cfg, sources)
                me = min(cfg.R // 2, sources - 1)
                own = np.bincount(w.K.reshape(-1), minlength=cfg.E)
                rows = int(M.astype(np.int64).sum() - M[me].sum() + own.sum())
                extra = dict(source_count=to_device(M), rank_id=me, window_rows=rows)
            layer = MoeLayer(cfg.T, cfg.H, cfg.k, cfg.E, cfg.R, dtype=cfg.dtype, schedule=schedule, **extra)
            xd, kd, wd = to_device(w.X), to_device(w.K), to_device(w.W)
            layer.dispatch(xd, kd)
            standin_expert(layer, to_device(w.scale))
            self.layers.append(layer), self.x.append(xd), self.k.append(kd), self.w.append(wd)
            if quant:     # e4m3 codes and row scales replace the bf16 window on the dispatch side
                self.wq.append(torch.empty((layer.rows, cfg.H), dtype=torch.uint8, device="cuda"))
                self.ws.append(torch.empty((layer.rows,), dtype=torch.float32, device="cuda"))
        torch.cuda.synchronize()
        self.schedule = self.layers[0].schedule
        self.bound = None

    def bind(self):
        """Pre-marshalled dispatch/combine calls per buffer set (see MoeLayer.bind)."""
        self.bound = [L.bind(self.x[j], self.k[j], self.w[j]) for j, L in enumerate(self.layers)]

    def step_bound(self, i):
        d, c = self.bound[i % self.n]
        d()
        c()

    def step(self, i):
        j = i % self.n
        L = self.layers[j]
        if self.quant:
            if L.schedule == self.moe.MOE_SCHEDULE_PREFILL:
                self.moe.moe_plan(L.shape, self.k[j], L._plan_struct)
            self.dispatch_only(i)
        else:
            L.dispatch(self.x[j], self.k[j])
        L.combine(self.w[j])

    def step_reuse(self, i):
        """Dispatch + combine with the plan left by an earlier call on the same routing (explicit schedule
        without moe_plan): the analogue of a cached mode for repeated calls with identical routing."""
        self.dispatch_only(i)
        self.layers[i % self.n].combine(self.w[i % self.n])

    def plan_only(self, i):
        j = i % self.n
        L = self.layers[j]
        self.moe.moe_plan(L.shape, self.k[j], L._plan_struct)

    def dispatch_only(self, i):
        j = i % self.n
        L = self.layers[j]
        if self.quant:
            self.moe.moe_dispatch_quant(L.shape, self.x[j], self.k[j], L._plan_struct, self.wq[j], self.ws[j])
        else:
            self.moe.moe_dispatch(L.shape, self.x[j], self.k[j], L._plan_struct, L.window)

    def combine_only(self, i):
        j = i % self.n
        self.layers[j].combine(self.w[j])


def graph_time_ms(fn, n_calls, replays):
    """Captures fn(0..n_calls-1) into one HIP graph and returns the average time per call over
    `replays` replays (launch cost is paid once per graph, as in a graph-captured serving loop)."""
    import torch
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(n_calls):
            fn(i)
    g.replay()
    torch.cuda.synchronize()
    return event_time_ms(lambda i: g.replay(), replays) / n_calls, g


def measure(cfg, steps, warmup, n_sets, use_graph=False, schedule=0, sources=1, quant=False, bound=False,
            reuse_plan=False, graph_too=False):
    import paper_2605_06055_amd as moe
    s = Sets(cfg, n_sets, schedule, sources, quant)
    if reuse_plan:                       # the constructor has planned every buffer set once
        assert s.schedule == moe.MOE_SCHEDULE_PREFILL and not quant
        s.step = s.step_reuse
    for i in range(warmup):
        s.step(i)
    n_pct = max(50, min(steps, 200))                  # layers whose wall time is taken one by one
    if use_graph:
        per_graph = max(n_sets, 20)
        ms, g = graph_time_ms(s.step, per_graph, max(1, steps // per_graph))
        pct = event_percentiles_us(lambda i: g.replay(), max(10, n_pct // per_graph), per_call=per_graph)
        pct["of"] = f"whole replays of the {per_graph}-layer graph, divided by {per_graph}"
    elif bound and not quant:
        s.bind()
        ms = event_time_ms(s.step_bound, steps)
        pct = event_percentiles_us(s.step_bound, n_pct)
        pct["of"] = "single layers, each between its own pair of events, launched back to back"
    else:
        ms = event_time_ms(s.step, steps)
        pct = event_percentiles_us(s.step, n_pct)
        pct["of"] = "single layers, each between its own pair of events, launched back to back"
    res = {"wall_us_per_layer": pct, "ms_per_step": ms, "us_per_layer": ms * 1e3, "gbs": cfg.payload_bytes / (ms * 1e-3) / 1e9,
           "schedule": "decode" if s.schedule == moe.MOE_SCHEDULE_DECODE else "prefill", "buffer_sets": n_sets,
           "launch": "hip graph replay" if use_graph else ("eager, pre-marshalled calls" if bound else "eager")}
    half = cfg.T * cfg.H * cfg.elem_bytes * (1 + cfg.k)           # bytes of dispatch alone == combine alone
    kern = {}
    if s.schedule == moe.MOE_SCHEDULE_PREFILL and not reuse_plan:
        kern["plan_us"] = event_time_ms(s.plan_only, steps) * 1e3
    if use_graph:
        per_graph = max(n_sets, 20)
        if "plan_us" in kern:
            kern["plan_us"] = graph_time_ms(s.plan_only, per_graph, max(1, steps // per_graph))[0] * 1e3
        kern["dispatch_us"] = graph_time_ms(s.dispatch_only, per_graph, max(1, steps // per_graph))[0] * 1e3
        kern["combine_us"] = graph_time_ms(s.combine_only, per_graph, max(1, steps // per_graph))[0] * 1e3
    else:
        kern["dispatch_us"] = event_time_ms(s.dispatch_only, steps) * 1e3
        kern["combine_us"] = event_time_ms(s.combine_only, steps) * 1e3
        # The same calls inside plan -> dispatch -> combine sequences, each between its own events: a kernel
        # then runs in the cache state the sequence leaves it (a loop of dispatches alone finds X in the
        # Infinity Cache whenever it fits), at the price of an event-to-event gap of a few microseconds
        # that these figures include.
        import torch
        calls = ([s.plan_only] if "plan_us" in kern else []) + [s.dispatch_only, s.combine_only]
        names = (["plan_us"] if "plan_us" in kern else []) + ["dispatch_us", "combine_us"]
        n = max(20, min(steps, 200))
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(n)]
        torch.cuda.synchronize()
        for i, e in enumerate(ev):
            e[0].record()
            for c, call in enumerate(calls):
                call(i)
                e[c + 1].record()
        torch.cuda.synchronize()
        res["kernels_in_sequence"] = {name: round(sum(e[c].elapsed_time(e[c + 1]) for e in ev) / n * 1e3, 2)
                                      for c, name in enumerate(names)}
    kern["dispatch_gbs"] = half / kern["dispatch_us"] / 1e3
    kern["combine_gbs"] = half / kern["combine_us"] / 1e3
    res["kernels"] = kern
    res["half_bytes"] = half
    if graph_too and not use_graph:
        # the same layers as one captured graph (kernel nodes only), replayed: what a serving loop that
        # captures its layers would see (no host launch work between the kernels)
        per_graph = max(n_sets, 40)          # enough layers per replay that the replay's own launch cost vanishes
        gms, g = graph_time_ms(s.step, per_graph, max(3, steps // per_graph))
        res["us_per_layer_graph"] = gms * 1e3
        del g
        if s.schedule == moe.MOE_SCHEDULE_PREFILL and n_sets == 1 and not quant:
            # The steps above all read the same X, which the Infinity Cache then still holds from the layer before
            # (as it would hold a tensor that the preceding operator has just written).  The same layers with X
            # rotating through 8 copies (more than the cache holds): every dispatch fetches its rows from HBM.
            xs = [s.x[0]] + [s.x[0].clone() for _ in range(7)]
            L = s.layers[0]

            nbytes = xs[0].numel() * xs[0].element_size()

            def step_x_cold(i, hint=False):
                if hint:        # moe_plan_t.prefetch: the plan pulls this X into the caches while it runs
                    L._plan_struct.prefetch, L._plan_struct.prefetch_bytes = xs[i % 8].data_ptr(), nbytes
                moe.moe_plan(L.shape, s.k[0], L._plan_struct)
                moe.moe_dispatch(L.shape, xs[i % 8], s.k[0], L._plan_struct, L.window)
                L.combine(s.w[0])
            step_x_cold(0)
            n_cold = max(16, steps // 16 * 16)
            res["us_per_layer_x_cold"] = event_time_ms(step_x_cold, n_cold) * 1e3
            res["us_per_layer_x_cold_prefetch"] = event_time_ms(lambda i: step_x_cold(i, True), n_cold) * 1e3
            L._plan_struct.prefetch, L._plan_struct.prefetch_bytes = xs[0].data_ptr(), nbytes
            res["us_per_layer_prefetch_x_warm"] = event_time_ms(s.step, n_cold) * 1e3
            L._plan_struct.prefetch, L._plan_struct.prefetch_bytes = None, 0
            del xs
    return res


def copy_ceiling():
    """Practical streaming roofs of the box, for context next to the 8 TB/s peak: a device-to-device
    memcpy of 1 GiB and the library's own 16-byte copy (dispatch with k = 1 and one expert is a plain
    row copy: 0.94 GB read + 0.94 GB written).  Bytes counted = read + written."""
    import torch
    import paper_2605_06055_amd as moe
    from paper_2605_06055_amd.layer import MoeLayer
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    ms = event_time_ms(lambda i: dst.copy_(src), 20)
    out = {"dtod_memcpy_GBps": round(2 * n / ms / 1e6, 1)}
    del src, dst
    T, H = 65536, 7168
    L = MoeLayer(T, H, 1, 1, 1, schedule=moe.MOE_SCHEDULE_PREFILL, separate_expert_out=False)
    x = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    kd = torch.zeros((T, 1), dtype=torch.int32, device="cuda")
    L.dispatch(x, kd)
    ms = event_time_ms(lambda i: moe.moe_dispatch(L.shape, x, kd, L._plan_struct, L.window), 20)
    out["own_copy_kernel_GBps"] = round(2 * T * H * 2 / ms / 1e6, 1)
    return out


def mix_ceilings(cfg, iters=30):
    """What the memory system sustains for the two access mixes of the path at this workload's shape,
    measured with plain kernels that share nothing with the library (ceilings/stream_mix.hip):
    8 reads : 1 write (combine's mix) and 1 read : 8 writes (dispatch's mix) of 16-byte vectors, once with
    purely sequential rows and once with the rows scattered over the expert blocks exactly as this workload's
    routing scatters them; plus read-only and write-only streams.  How workgroups are mapped to the data
    matters as much as the mix, so each figure is the best of several launch forms (named beside it).
    GB/s over bytes read + written; loops of identical launches, i.e. the conditions of `kernels`."""
    import numpy as np
    import torch
    import ceilings
    import workloads as wl
    T, H, k = cfg.T, cfg.H, cfg.k
    assert k == 8
    cols = H * cfg.elem_bytes // 16
    big = torch.empty((T * k, H), dtype=torch.bfloat16, device="cuda").fill_(1.0)
    small = torch.empty((T, H), dtype=torch.bfloat16, device="cuda").fill_(2.0)
    K = wl.draw_routing(cfg, np.random.default_rng(cfg.seed)).reshape(-1)
    order = np.argsort(K, kind="stable")                      # branches in window-row order (expert blocks)
    scattered = np.empty(T * k, np.int32)
    scattered[order] = np.arange(T * k, dtype=np.int32)
    tables = {"sequential": torch.arange(T * k, dtype=torch.int32, device="cuda"),
              "scattered": torch.from_numpy(scattered).cuda()}
    for table in tables.values():
        ceilings._check_table(table, T * k)
    total = (1 + k) * T * H * cfg.elem_bytes
    out = {"bytes_per_launch": total,
           "forms": "gather: (workgroup size, nontemporal loads, mapping); scatter: (table entries per workgroup, "
                    "nontemporal loads, mapping); mapping 0 = (row, chunk) order, 1 = XCD-affine column slices, "
                    "2 = each XCD walks a contiguous eighth, 3 = one 512-thread workgroup per compute unit that holds "
                    "the results of 28 units per thread back until their loads are done; stores nontemporal"}
    for name, fn, forms, src, dst in (("read8_write1", ceilings.gather8, ceilings.GATHER_FORMS, big, small),
                                      ("read1_write8", ceilings.scatter8, ceilings.SCATTER_FORMS, small, big)):
        for tname, table in tables.items():
            best, best_form = None, None
            for form in forms:
                if form[2] == 3 and cols % 64:
                    continue
                call = lambda i: fn(form, src, table, dst, T, cols)
                call(0)
                ms = event_time_ms(call, iters)
                if best is None or ms < best:
                    best, best_form = ms, form
            out[f"{name}_{tname}_us"] = round(best * 1e3, 2)
            out[f"{name}_{tname}_GBps"] = round(total / best / 1e6, 1)
            out[f"{name}_{tname}_form"] = list(best_form)
    sink = torch.zeros(16, dtype=torch.int32, device="cuda")
    for nt in (True, False):
        ceilings.read(big, sink, nt)
        ms = event_time_ms(lambda i: ceilings.read(big, sink, nt), iters)
        out["read_only_GBps"] = max(out.get("read_only_GBps", 0), round(big.numel() * 2 / ms / 1e6, 1))
        ceilings.write(big, nt)
        ms = event_time_ms(lambda i: ceilings.write(big, nt), iters)
        out["write_only_GBps"] = max(out.get("write_only_GBps", 0), round(big.numel() * 2 / ms / 1e6, 1))
    # the serial model: reads and writes share one bus, so a mix cannot beat bytes_read / read_only + bytes_written / write_only
    rd, wr = out["read_only_GBps"] * 1e3, out["write_only_GBps"] * 1e3      # bytes per microsecond
    big_b, small_b = k * T * H * cfg.elem_bytes, T * H * cfg.elem_bytes
    out["read8_write1_serial_model_us"] = round(big_b / rd + small_b / wr, 2)
    out["read1_write8_serial_model_us"] = round(small_b / rd + big_b / wr, 2)
    return out


def cpu_baseline(cfg, budget_s=10.0):
    """The oracle as it stands on a bounded sample of the same workload: single thread (the headline
    figure) and, beside it, the same source built with OpenMP so that the token loops of dispatch and
    combine use every host core (the plan stays serial)."""
    import oracle
    import workloads as wl
    T = min(cfg.T, 4096)                           # the whole headline batch; a slice of the larger workloads
    sub = cfg.with_(T=T)
    w = wl.make(sub)

    def timed(budget):
        reps, spent = 0, 0.0
        while reps < 1 or (spent < budget and reps < 50):
            t0 = time.perf_counter()
            pl = oracle.plan(w.K, sub.E, sub.R)
            window = oracle.dispatch(w.X, pl.row_map, pl.window_rows)
            oracle.combine(window, w.W, pl.row_map)
            spent += time.perf_counter() - t0
            reps += 1
        return spent / reps, reps

    per, reps = timed(budget_s)
    with oracle.all_cores():
        threads = oracle.threads()
        per_all, reps_all = timed(budget_s / 2)
    return {"value": sub.payload_bytes / per / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": (f"the whole batch of {T} tokens" if T == cfg.T else f"first {T} tokens of the workload")
                      + f" (plan+dispatch+combine, identity expert), {reps} repetitions, {per * 1e3:.1f} ms each",
            "all_cores": {"value": round(sub.payload_bytes / per_all / 1e9, 3), "unit": "GB/s", "cores": threads,
                          "sample": f"same sample, {reps_all} repetitions, {per_all * 1e3:.1f} ms each"},
            "host_cpus": os.cpu_count()}


def traffic_for(kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc (committed summary of two counter runs,
    scaled by a plain copy of known size), or None when no summary covers this kernel and workload.
    Returns (bytes, where the figure comes from)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(path))
        return table[kernel]["total_bytes"], table.get("_source", "profiles/hbm_traffic.json")
    except (OSError, ValueError, KeyError):
        return None, None


def compact(res, cfg):
    """One workload's figures for the JSON line."""
    pct = res["wall_us_per_layer"]
    out = {"workload": DESCR[cfg.name], "us_per_layer": round(res["us_per_layer"], 2),
           "value": round(res["gbs"], 1), "unit": "GB/s",
           "frac_of_hbm_peak": round(res["gbs"] / HBM_PEAK_GBS, 4),
           "us_per_layer_p50": pct["p50"],
           "frac_of_hbm_peak_p50": round(cfg.payload_bytes / pct["p50"] / 1e3 / HBM_PEAK_GBS, 4),
           "kernels": rounded(res["kernels"]), "kernels_in_sequence": res.get("kernels_in_sequence")}
    if "us_per_layer_graph" in res:
        out["us_per_layer_graph"] = round(res["us_per_layer_graph"], 2)
        out["frac_of_hbm_peak_graph"] = round(cfg.payload_bytes / res["us_per_layer_graph"] / 1e3 / HBM_PEAK_GBS, 4)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="prefill", choices=sorted(DESCR))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode T=128 leg of the headline run")
    ap.add_argument("--no-others", action="store_true", help="skip the skewed and wide prefill workloads")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the streaming-copy ceiling measurement")
    ap.add_argument("--decode-sweep", action="store_true",
                    help="also time decode layers at the paper's Table 2 points: hidden 4096 and 7168, "
                         "batch 16..144 (HIP graph replay, cold buffers); printed to stderr and added to the JSON")
    ap.add_argument("--prefill-sweep", action="store_true",
                    help="also time prefill layers (explicit plan) at 1024..16384 tokens of the H=7168 layer, the "
                         "token axis of the paper's prefill figure, with the bf16 and the quantised dispatch")
    ap.add_argument("--quant", action="store_true",
                    help="also time prefill T=4096 and decode T=128 with the row-wise quantised dispatch "
                         "(FP8 E4M3 codes + fp32 row scales on the dispatch side, bf16 combine)")
    ap.add_argument("--multi-source", type=int, default=0, metavar="S",
                    help="also time prefill T=4096 and decode T=128 as one of S source ranks (count matrix M given, "
                         "windows hold the blocks of all S sources)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain elementwise copy of known size (512 MiB read + 512 MiB written, "
                         "torch.mul(src, 1, out=dst)) so that rocprofv3 --pmc counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the dispatch/combine path; this build has no multi-GPU "
              "path (no collectives are part of it). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    import paper_2605_06055_amd as moe
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    moe.load_library()
    torch.cuda.set_device(0)

    if args.calibrate:
        src = torch.ones(128 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    cfg = wl.CONFIGS[args.workload]
    n_sets = 20 if cfg.payload_bytes < 512e6 else 1
    main_res = measure(cfg, args.steps, args.warmup, n_sets, graph_too=True)
    log(f"[{args.workload}] {json.dumps(main_res)}")

    # The dominant kernel and its duration come from plan -> dispatch -> combine sequences (each call between
    # its own HIP events on the launch stream), i.e. in the cache state the layer really leaves; a loop of
    # identical launches (`kernels`) can flatter a kernel whose input stays in the Infinity Cache.
    kern = main_res["kernels"]
    seq = main_res.get("kernels_in_sequence") or {k: v for k, v in kern.items() if k.endswith("_us")}
    dom = "moe_combine" if seq["combine_us"] >= seq["dispatch_us"] else "moe_dispatch"
    dom_us = max(seq["combine_us"], seq["dispatch_us"])
    achieved = main_res["half_bytes"] / dom_us / 1e3
    traffic, traffic_source = traffic_for(f"{dom}:{args.workload}")
    head = compact(main_res, cfg)
    out = {
        "metric": "dispatch+combine effective HBM GB/s", "value": round(main_res["gbs"], 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(main_res["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",       # arithmetic of the path: fp32 multiply-add in combine (dispatch is a byte copy, the plan int32)
        "data": "synthetic",
        "config": {"workload": DESCR[args.workload], "schedule": main_res["schedule"], "storage": "bf16",
                   "payload_bytes_per_step": cfg.payload_bytes, "buffer_sets": n_sets},
        "us_per_layer": head["us_per_layer"],
        "wall_us_per_layer": main_res["wall_us_per_layer"],
        "frac_of_hbm_peak": head["frac_of_hbm_peak"],
        "frac_of_hbm_peak_p50": head["frac_of_hbm_peak_p50"],
        "us_per_layer_graph": head.get("us_per_layer_graph"),
        "frac_of_hbm_peak_graph": head.get("frac_of_hbm_peak_graph"),
        "x_cold": None if "us_per_layer_x_cold" not in main_res else {
            "us_per_layer": round(main_res["us_per_layer_x_cold"], 2),
            "frac_of_hbm_peak": round(cfg.payload_bytes / main_res["us_per_layer_x_cold"] / 1e3 / HBM_PEAK_GBS, 4),
            "what": "the same layers with X rotating through 8 copies, so that no dispatch finds its token rows in "
                    "the Infinity Cache (the headline steps re-read one X, as after an operator that has just written it)",
            "us_per_layer_with_plan_prefetch": round(main_res["us_per_layer_x_cold_prefetch"], 2),
            "frac_of_hbm_peak_with_plan_prefetch": round(cfg.payload_bytes / main_res["us_per_layer_x_cold_prefetch"]
                                                         / 1e3 / HBM_PEAK_GBS, 4),
            "plan_prefetch": "moe_plan_t.prefetch = X: spare workgroups of the plan read X while the plan runs; the "
                             "headline does not use it, and with X warm it costs: us_per_layer_warm_with_plan_prefetch",
            "us_per_layer_warm_with_plan_prefetch": round(main_res["us_per_layer_prefetch_x_warm"], 2)},
        "kernels": rounded(kern),
        "kernels_in_sequence": main_res.get("kernels_in_sequence"),
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "duration_us": round(dom_us, 2),
                     "duration_from": "HIP events around the call inside plan->dispatch->combine sequences "
                                      "(includes the event-to-event gap); `kernels` holds back-to-back loops",
                     "traffic": traffic, "traffic_source": traffic_source},
    }
    if not args.no_ceiling:
        out["copy_ceiling"] = copy_ceiling()
        out["frac_of_copy_ceiling"] = round(main_res["gbs"] / max(out["copy_ceiling"].values()), 4)
        mc = mix_ceilings(cfg)
        log(f"[mix ceilings] {json.dumps(mc)}")
        out["mix_ceiling"] = mc
        # like with like: the library's kernels in loops of identical launches against the plain kernels in
        # the same kind of loop, for the scattered rows of this routing and for purely sequential rows
        out["frac_of_mix_ceiling"] = {
            "dispatch_vs_read1_write8_scattered": round(mc["read1_write8_scattered_us"] / kern["dispatch_us"], 4),
            "combine_vs_read8_write1_scattered": round(mc["read8_write1_scattered_us"] / kern["combine_us"], 4),
            "dispatch_vs_read1_write8_sequential": round(mc["read1_write8_sequential_us"] / kern["dispatch_us"], 4),
            "combine_vs_read8_write1_sequential": round(mc["read8_write1_sequential_us"] / kern["combine_us"], 4)}
    if args.workload == "prefill" and not args.no_others:
        # the other two prefill workloads of the configuration list, one compact entry each
        out["workloads"] = {}
        for name in ("skewed", "wide"):
            c = wl.CONFIGS[name]
            r = measure(c, max(10, args.steps // 4), max(2, args.warmup // 4), 1)
            log(f"[{name}] {json.dumps(r)}")
            out["workloads"][name] = compact(r, c)
            del r
            torch.cuda.empty_cache()
    if args.workload == "prefill" and not args.no_decode:
        dcfg = wl.CONFIGS["decode"]
        d = measure(dcfg, max(args.steps, 400), args.warmup, 20, use_graph=True)
        de = measure(dcfg, max(args.steps, 400), args.warmup, 20, use_graph=False, bound=True)
        dw = measure(dcfg, max(args.steps, 400), args.warmup, 1, use_graph=True)
        log(f"[decode, graph replay, one buffer set (warm cache)] {json.dumps(dw)}")
        dr = measure(dcfg, max(args.steps, 400), args.warmup, 20, use_graph=True, schedule=1, reuse_plan=True)
        log(f"[decode, graph replay, plan reused] {json.dumps(dr)}")
        log(f"[decode, graph replay] {json.dumps(d)}")
        log(f"[decode, eager launches from Python, pre-marshalled] {json.dumps(de)}")
        out["decode"] = {"workload": DESCR["decode"], "us_per_layer": round(d["us_per_layer"], 2),
                         "value": round(d["gbs"], 1), "unit": "GB/s",
                         "frac_of_hbm_peak": round(d["gbs"] / HBM_PEAK_GBS, 4),
                         "frac_of_hbm_peak_p50": round(dcfg.payload_bytes / d["wall_us_per_layer"]["p50"] / 1e3
                                                       / HBM_PEAK_GBS, 4),
                         "buffer_sets": d["buffer_sets"],
                         "launch": "one HIP graph of 20 layers replayed (a layer is 2 kernels of ~5 us)",
                         "wall_us_per_layer": d["wall_us_per_layer"],
                         "us_per_layer_warm": round(dw["us_per_layer"], 2),
                         "warm": "the same graph on ONE buffer set (33 MB, resident in the Infinity Cache): not an "
                                 "HBM figure, shown for contrast only",
                         "us_per_layer_plan_reused": round(dr["us_per_layer"], 2),
                         "plan_reused": "cold buffers, same graph replay, but the routing plan of an earlier call on "
                                        "identical routing is reused (dispatch reads the stored row map): a cached "
                                        "mode for repeated routing, not the figure for fresh routing",
                         "us_per_layer_eager": round(de["us_per_layer"], 2),
                         "eager_launch": "kernel by kernel from Python with pre-marshalled ctypes arguments "
                                         "(MoeLayer.bind); marshalling per call would cost ~7 us per launch",
                         "cache": "cold: 20 disjoint buffer sets (660 MB) rotated so no step finds its lines in "
                                  "the 256 MB Infinity Cache",
                         "kernels": rounded(d["kernels"])}
        ddom = "moe_dispatch" if d["kernels"]["dispatch_us"] >= d["kernels"]["combine_us"] else "moe_combine"
        dus = max(d["kernels"]["dispatch_us"], d["kernels"]["combine_us"])
        dtraffic, dsource = traffic_for(f"{ddom}:decode")
        out["decode"]["roofline"] = {"bound": "hbm", "kernel": ddom, "achieved": round(d["half_bytes"] / dus / 1e3, 1),
                                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                     "frac": round(d["half_bytes"] / dus / 1e3 / HBM_PEAK_GBS, 4),
                                     "duration_us": round(dus, 2),
                                     "duration_from": "graph replay of 20 launches of the kernel alone on cold buffers",
                                     "traffic": dtraffic, "traffic_source": dsource}
    if args.quant:
        pc, dc = wl.CONFIGS["prefill"], wl.CONFIGS["decode"]
        qp = measure(pc, args.steps, args.warmup, 1, quant=True)
        qd = measure(dc, max(args.steps, 400), args.warmup, 20, use_graph=True, quant=True)
        log(f"[prefill, quantised dispatch] {json.dumps(qp)}")
        log(f"[decode, quantised dispatch, graph replay] {json.dumps(qd)}")

        def qbytes(c):      # X read once as bf16; codes (1 byte) and a 4-byte scale written per routed row
            return c.T * c.H * 2 + c.N * (c.H + 4)
        out["quantised_dispatch"] = {
            "format": "OCP FP8 E4M3 codes + fp32 scale per row (amax/448)",
            "prefill": {"us_per_layer": round(qp["us_per_layer"], 2),
                        "dispatch_us": round(qp["kernels"]["dispatch_us"], 2), "dispatch_bytes": qbytes(pc),
                        "dispatch_GBps": round(qbytes(pc) / qp["kernels"]["dispatch_us"] / 1e3, 1),
                        "combine_us": round(qp["kernels"]["combine_us"], 2)},
            "decode": {"us_per_layer": round(qd["us_per_layer"], 2),
                       "dispatch_us": round(qd["kernels"]["dispatch_us"], 2), "dispatch_bytes": qbytes(dc),
                       "dispatch_GBps": round(qbytes(dc) / qd["kernels"]["dispatch_us"] / 1e3, 1),
                       "combine_us": round(qd["kernels"]["combine_us"], 2)}}
    if args.multi_source > 1:
        S = args.multi_source
        mp = measure(wl.CONFIGS["prefill"], args.steps, args.warmup, 1, sources=S)
        md = measure(wl.CONFIGS["decode"], max(args.steps, 400), args.warmup, 20, use_graph=True, sources=S)
        log(f"[prefill as one of {S} sources] {json.dumps(mp)}")
        log(f"[decode as one of {S} sources, graph replay] {json.dumps(md)}")
        out["multi_source"] = {"sources": S,
                               "prefill_us_per_layer": round(mp["us_per_layer"], 2),
                               "prefill_kernels": rounded(mp["kernels"]),
                               "decode_us_per_layer": round(md["us_per_layer"], 2),
                               "decode_kernels": rounded(md["kernels"])}
    if args.decode_sweep:
        sweep = []
        for H in (4096, 7168):
            for T in (16, 32, 64, 80, 128, 144):
                c = wl.CONFIGS["decode"].with_(name=f"decode_T{T}_H{H}", T=T, H=H)
                n_sets = max(20, int(600e6 // c.payload_bytes))
                r = measure(c, 800, 5, min(n_sets, 200), use_graph=True)
                row = {"H": H, "T": T, "us_per_layer": round(r["us_per_layer"], 2),
                       "dispatch_us": round(r["kernels"]["dispatch_us"], 2),
                       "combine_us": round(r["kernels"]["combine_us"], 2), "GBps": round(r["gbs"], 1)}
                log(f"[decode sweep] {json.dumps(row)}")
                sweep.append(row)
        out["decode_sweep"] = sweep
    if args.prefill_sweep:
        sweep = []
        for T in (1024, 2048, 4096, 8192, 16384):
            c = wl.CONFIGS["prefill"].with_(name=f"prefill_T{T}", T=T)
            n_sets = 4 if c.payload_bytes < 400e6 else 1          # keep the working set well over 256 MB
            r = measure(c, 100, 5, n_sets, schedule=1)
            q = measure(c, 100, 5, n_sets, schedule=1, quant=True)
            row = {"T": T, "us_per_layer": round(r["us_per_layer"], 1), "GBps": round(r["gbs"], 1),
                   "plan_us": round(r["kernels"]["plan_us"], 1), "dispatch_us": round(r["kernels"]["dispatch_us"], 1),
                   "combine_us": round(r["kernels"]["combine_us"], 1),
                   "quant_dispatch_us": round(q["kernels"]["dispatch_us"], 1)}
            log(f"[prefill sweep] {json.dumps(row)}")
            sweep.append(row)
        out["prefill_sweep"] = sweep
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
        out["cpu_baseline"]["value"] = round(out["cpu_baseline"]["value"], 3)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
