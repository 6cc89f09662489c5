"""The benchmark's output contract, checked on the GPU: bench.py runs as a child process (shortened)
and must print one JSON line with the throughput fields, the roofline and the per-layer table."""

import pytest

pytestmark = pytest.mark.gpu


def test_bench_prints_one_json_line_with_the_contract_fields():
    # the default benchmark, shortened: one JSON line on stdout with the throughput fields, the
    # roofline of the dominant kernel and the per-layer table
    import json
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "5", "--warmup", "2", "--no-cpu-baseline", "--no-70b", "--no-lm-head", "--no-qwen"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
                "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "GB/s" and d["value"] > 0
    assert "workload" in d["config"] and d["vs_baseline"] is None and d["cpu_baseline"] is None  # --no-cpu-baseline
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and 0.2 < rf["frac"] < 1.0
    # the batch sweep of the 8B gate/up and down projections rides in the same line
    assert {(r["layer"], r["M"], r["fmt"]) for r in d["batch_sweep"]} == {(n, m, f) for n in ("gate_up", "down") for m in (1, 2, 4, 8, 16, 32)
                                                                       for f in ("fp5.33-e2m3", "fp4.25-e2m2")}
    assert all(r["us"] > 0 and (r["us_static_ws"] or 1) > 0 and r["speedup_vs_best_fp16"] > 0 for r in d["batch_sweep"])
    assert d["llama70b"] is None and d["lm_head"] is None and d["qwen_down"] is None  # --no-70b --no-lm-head --no-qwen
    assert {(l["layer"], l["fmt"]) for l in d["layers"]} == {(n, f) for n in ("qkv", "o", "gate_up", "down") for f in ("fp5.33-e2m3", "fp4.25-e2m2")}
