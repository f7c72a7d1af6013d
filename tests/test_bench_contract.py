"""The command-line contract of bench.py: one GPU only, and one JSON line with the fields the
measurement is read from."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         cwd=ROOT, timeout=300)
    assert res.returncode != 0
    assert "single-GPU" in (res.stderr + res.stdout) and "--gpus 1" in (res.stderr + res.stdout)


@pytest.mark.gpu
def test_default_workload_prints_one_json_line_with_roofline_and_comparison():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "2",
                          "--no-cpu-baseline"], capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["unit"] == "TFLOP/s" and d["dtype"] == "bf16" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["config"]["workload"].startswith("cfg3") and "model" not in d["config"]
    assert d["value"] > 100 and abs(d["ms_per_step"] - (d["fwd_ms"] + d["bwd_dkdv_ms"] + d["bwd_dq_ms"])) < 0.2 * d["ms_per_step"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-6 and 0.2 < r["frac"] < 1.0
    # the softmax comparison is part of the default run: both methods hand-pinned, and the twins
    for key in ("softmax_fwd_ms", "softmax_bwd_ms", "softmax_bwd_compiler_scheduled_ms", "sigmoid_bwd_compiler_scheduled_ms",
                "fwd_time_ratio_like_for_like", "bwd_time_ratio_like_for_like", "bwd_time_ratio_like_for_like_compiler_scheduled"):
        assert d[key] > 0, key
    assert d["fwd_time_ratio_like_for_like"] < 1.0          # the forward is where the method wins
    assert d["softmax_bwd_ms"] < 0.7 * d["softmax_bwd_compiler_scheduled_ms"]   # the pinned softmax backward is in use
