"""Host-side checks of bench.py that need no GPU: the multi-GPU refusal, the byte accounting and the
bounded oracle baseline."""
import json
import os
import subprocess
import sys

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in (res.stderr + res.stdout)
    assert not res.stdout.strip().startswith("{")           # no result line is printed


def test_payload_accounting_is_the_algorithmic_bytes_of_a_step():
    for name, cfg in wl.CONFIGS.items():
        b = cfg.elem_bytes
        assert cfg.payload_bytes == 2 * cfg.T * cfg.H * b * (1 + cfg.k), name
    assert wl.CONFIGS["prefill"].payload_bytes == 1_056_964_608
    assert wl.CONFIGS["decode"].payload_bytes == 33_030_144


def test_committed_traffic_summary_covers_the_named_workloads():
    d = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
    for wlname in ("prefill", "decode", "skewed", "wide"):
        for kern in ("moe_dispatch", "moe_combine"):
            e = d[f"{kern}:{wlname}"]
            cfg = wl.CONFIGS[wlname]
            assert e["algorithmic_bytes"] == cfg.payload_bytes // 2
            assert e["total_bytes"] == e["fetch_bytes"] + e["write_bytes"]
            # no wasted re-reads.  The counters count what leaves L2, whether the Infinity Cache or HBM serves it: the
            # dispatch along the order list re-fetches X slices that L2 dropped (1.6 x X, 7 % of the launch's bytes)
            assert 0.99 <= e["total_bytes"] / e["algorithmic_bytes"] <= (1.08 if f"{kern}:{wlname}" == "moe_dispatch:prefill" else 1.05)
            got, source = bench.traffic_for(f"{kern}:{wlname}")
            assert got == e["total_bytes"] and source == d["_source"]
    assert bench.traffic_for("moe_combine:no such workload") == (None, None)


def test_cpu_baseline_runs_the_oracle_on_a_bounded_sample():
    cfg = wl.CONFIGS["prefill"].with_(T=64, H=256)
    r = bench.cpu_baseline(cfg, budget_s=0.2)
    assert r["kind"] == "oracle" and r["cores"] == 1 and r["unit"] == "GB/s" and r["value"] > 0
    assert r["all_cores"]["cores"] >= 1 and r["all_cores"]["value"] > 0
