"""bench.py prints ONE JSON line with the agreed fields (run with few steps);
the line's own parity flag must be true."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_default_bench_line(gpu):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["unit"] == "GB/s" and d["data"] == "synthetic"
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["dtype"] == "u32"
    assert "workload" in d["config"] and "model" not in d["config"]
    assert d["parity_vs_oracle"] is True
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel"):
        assert key in roof, key
    assert roof["kernel"] == "k_gather" and 0.5 < roof["frac"] <= 1.05
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert abs(d["value"] - roof["achieved"]) / d["value"] < 0.02       # wall clock and HIP events agree
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0 and cpu["sample"]
    assert len(cpu["note"]) < 256 and cpu["unit"] == "useful GB/s" and cpu["job_seconds"] > 0
    par = d["cpu_baseline_all_cores"]
    assert par["cores"] >= 1 and par["value"] > 0 and par["job_seconds"] > 0
    job = d["job_seconds"]
    assert job["gpu_paging"] > 0 and job["cpu_oracle_1_core"] > 0 and job["gpu_zero_copy"] > 0
    assert any(k.startswith("cpu_parallel_for_") for k in job)
    dd = d["dedup"]                                                      # wavefront dedup and arbitration, in numbers
    assert dd["wave_page_groups"] + dd["lanes_coalesced"] == dd["lane_accesses"] == d["config"]["indices"]
    assert dd["hits"] + dd["faults"] == dd["wave_page_groups"] and dd["lanes_per_group"] >= 1.0
    hp = d["hit_path"]                                                   # hits only, each leg with a roofline object of its own
    for leg in ("random_4KiB_pages", "random_64KiB_pages", "unit_stride_4KiB_pages", "unit_stride_64KiB_pages", "whole_pages_64KiB"):
        assert hp[leg]["parity"] and hp[leg]["new_faults"] == 0, leg
        assert hp[leg]["roofline"]["bound"] == "hbm" and 0 < hp[leg]["roofline"]["frac"] <= 1.0, leg
