"""The benchmark script's contract: one JSON line with the agreed fields; one GPU only."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


@pytest.mark.gpu
@pytest.mark.parametrize("extra", [[], ["--graph"], ["--optimizer", "momentum", "--combine"], ["--propagation", "gradient"]])
def test_bench_line_on_the_small_workload(extra):
    if extra:
        extra = [*extra, "--row-traffic", "0"]         # the child process that measures those figures: once is enough
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "tiny", "--steps", "3",
                        "--warmup", "1", *extra], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["value"] > 0 and d["vs_baseline"] is None
    assert d["config"]["workload"].startswith("tiny") and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    assert r["traffic"] is None                        # counters exist for the default workload only
    by_distance = d["ceilings"]["row_traffic_by_distance"]
    if extra:
        assert by_distance is None
    else:                                              # read-modify-write of rows never beats reading them
        assert by_distance["read_write_GBps"] and by_distance["read_GBps"].keys() == by_distance["read_write_GBps"].keys()
        assert all(0 < by_distance["read_write_GBps"][g] < 1.05 * by_distance["read_GBps"][g] for g in by_distance["read_GBps"])
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1
