"""bench.py's contract: one JSON line with the agreed fields (GPU, on the smallest workload), and a refusal of
more than one GPU (CPU)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_fields():
    print("case bench.py on the smallest workload", flush=True)
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "C1", "--steps", "24", "--warmup", "4",
                        "--settle-ms", "5"], capture_output=True, text=True, timeout=240, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 24 and d["warmup"] == 4 and d["higher_is_better"] is True
    assert d["data"] == "synthetic" and d["vs_baseline"] is None and "workload" in d["config"]
    r = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel_ms", "kernel_launches_timed",
                "device_copy_ceiling_GBps"):
        assert key in r, key
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["kernel_launches_timed"] == 24
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    assert 0 < r["kernel_ms"] <= d["ms_per_step"] * 1.05           # the launches lie inside the timed region (two clocks)
    assert abs(d["value"] - 20 * 32 / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]      # T * B steps per step
    c = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample", "single_thread_value", "nproc", "cpu_model"):
        assert key in c, key
    assert c["kind"] == "oracle" and c["cores"] >= 1
