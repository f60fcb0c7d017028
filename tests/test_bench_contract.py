"""bench.py keeps its output contract: one JSON line with the fields the driver reads."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)


@pytest.mark.gpu
@pytest.mark.parametrize("launch", ["native", "hybrid", "graph", "native --refresh second-stream", "native --no-overlap",
                                    "eager"])
def test_bench_json_line_small_workload(launch):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "cfg1_llama_2k", "--layers", "3", "--steps", "12",
           "--warmup", "2", "--cpu-layers", "1", "--launch"] + launch.split()
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "roofline_partial", "copy_GBps", "read_GBps", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 12 and d["warmup"] == 2 and d["higher_is_better"] is False
    assert d["config"]["workload"] == "cfg1_llama_2k" and d["value"] > 0
    for block in ("roofline", "roofline_partial"):
        for key in ("bound", "kernel", "achieved", "peak", "unit", "frac", "traffic", "traffic_source", "avg_launch_us",
                    "algorithmic_bytes"):
            assert key in d[block], (block, key)
        assert d[block]["bound"] == "hbm" and 0 < d[block]["frac"] < 1
    assert d["copy_GBps"] > 0
    assert d["read_GBps"]["one_launch_1GiB"] > 0 and d["read_GBps"]["launches_of_full_attn_kv_bytes"] > 0
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in d["cpu_baseline"], key
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["value"] > 0
