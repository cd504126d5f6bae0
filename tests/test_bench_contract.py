"""The benchmark's command-line contract: more than one GPU is refused with a message (no GPU needed to see
that), and a run prints exactly one JSON line with the agreed keys (GPU)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_keys():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--configs", "1,1", "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["data"] == "synthetic" and "workload" in d["config"] and d["value"] > 0
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in d["roofline"], key
    assert abs(d["roofline"]["frac"] - d["roofline"]["achieved"] / d["roofline"]["peak"]) < 1e-9
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in d["cpu_baseline"], key
    assert d["cpu_baseline"]["kind"] == "oracle"
    assert d["attention_status_word"] == 0
    # median and minimum beside the mean, the same loop on one set of buffers, the reproducible mode
    for key in ("step_gpu_ms_median", "step_gpu_ms_min", "same_buffers"):
        assert key in d, key
    for key in ("kernel_ms_avg", "kernel_ms_median", "kernel_ms_min", "same_buffers", "fixed_split", "kernel"):
        assert key in d["roofline"], key
    assert d["roofline"]["kernel"].startswith("attn_gqa128_kernel<1,1>")
    # the other workloads ride in the same line, each with a roofline of its own
    assert set(d["per_config"]) == {"config1"} and "roofline" in d["per_config"]["config1"]
