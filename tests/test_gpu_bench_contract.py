"""The measurement script keeps its contract: one JSON line with the agreed keys on a small workload (run as a
child process, like the driver does), the roofline and CPU-baseline objects, parity of the timed output; more than
one GPU is refused (this build is for one)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args, timeout=300):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=timeout)


@pytest.mark.gpu
@pytest.mark.parametrize("workload,tries", [("csa256_b1_F64", 3), ("csa32_b1_F32", 0)])
def test_bench_line_on_a_small_workload(workload, tries):
    print(f"bench.py --workload {workload} --placement-tries {tries}", flush=True)
    res = _bench("--workload", workload, "--steps", "3", "--warmup", "1", "--placement-tries", str(tries))
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, res.stdout[-2000:]
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["unit"] == "GFLOP/s" and d["dtype"] == "f32" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["config"]["workload"] == workload and "model" not in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s" and "traffic" in r
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
    assert d["parity_max_err_over_tol"] <= 1.0           # the timed output, element by element against the oracle
    if tries:
        assert d["placement"]["arena_matrices"] >= 3 and d["placement"]["kept_ms"] > 0
    else:
        assert d["placement"] is None


def test_more_than_one_gpu_is_refused():
    res = _bench("--gpus", "2", timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr or "--gpus 1" in res.stderr
