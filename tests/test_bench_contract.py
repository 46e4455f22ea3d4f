"""bench.py's contract: refuses more than one GPU with a message (checked without a GPU); on a GPU,
a short run prints one JSON line with the fields the harness reads."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert run.returncode != 0
    assert "one-GPU" in run.stderr + run.stdout


@pytest.mark.gpu
def test_short_run_prints_the_json_line():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--log2d", "22", "--steps", "2", "--warmup", "1",
                          "--cpu-sample-log2", "18"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [l for l in run.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    r = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 2 and r["warmup"] == 1 and r["vs_baseline"] is None
    assert r["value"] > 0 and r["ms_per_step"] > 0 and "workload" in r["config"]
    rf = r["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert rf["traffic"] is None or isinstance(rf["traffic"], int)   # bytes per launch, null off the profiled workload
    assert set(r["per_b"]) == {str(b) for b in range(1, 9)}
    cb = r["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    for name in ("dq_norm", "dq_quantize_pack", "dq_unpack_dequant_reduce", "dq_norm_quantize_pack",
                 "dq_norm_quantize_pack_bracketed"):
        assert r["kernels"][name]["avg_ms"] > 0
