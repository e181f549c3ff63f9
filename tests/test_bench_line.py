"""bench.py's one JSON line, on one layer of the set with every extra: the fields of the contract, the
pattern the headline is quoted on, and the arithmetic that ties value, ms_per_step and the roofline together."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_bench_line_on_one_layer():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--layers", "1", "--steps", "3", "--warmup", "1",
                          "--no-cpu-baseline"], cwd=ROOT, capture_output=True, text=True, timeout=280)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [x for x in run.stdout.splitlines() if x.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["unit"] == "Gparams/s"
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "f32"
    cfg = d["config"]
    assert (cfg["n_keep"], cfg["m_group"], cfg["scale_segments"]) == (2, 4, 2) and "2:4" in cfg["workload"]
    params = 4 * 4096 * 4096 + 3 * 11008 * 4096
    assert f"{params} params" in cfg["workload"]
    assert d["value"] == pytest.approx(params / (d["ms_per_step"] * 1e-3) / 1e9, rel=1e-3)
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert r["frac"] == pytest.approx(r["achieved"] / r["peak"], abs=1e-4)
    assert r["achieved"] == pytest.approx(r["bytes_per_launch"] / (r["avg_launch_us"] * 1e-6) / 1e9, rel=1e-3)
    assert 0.3 < r["frac"] < 1.0
    assert r["traffic"] is None or 1.0 <= r["traffic"] / r["bytes_per_launch"] < 1.05
    # every extra ran (none of them replaced by a failure record)
    extra = d["extra"]
    for key in ("nm_select_GBs", "project_compress_GBs", "weight_scale_bf16_GBs", "mask_stats_GBs", "pattern_4of8",
                "pattern_1of2", "fp32_grads", "long_forms", "stream_probe"):
        assert key in extra and "failed" not in json.dumps(extra[key]), (key, extra.get(key))


def test_more_than_one_gpu_is_refused():
    # decided before anything touches the GPU: runs anywhere
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT, capture_output=True,
                         text=True, timeout=60)
    assert run.returncode != 0 and "one GPU" in run.stderr
