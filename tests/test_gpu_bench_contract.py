"""``bench.py`` on the GPU machine: one JSON line with the keys of the benchmark contract, the roofline and CPU-baseline
objects, the parity gate (the timed kernel's output against whole oracle heads) and a zero exit code; more than one
GPU is refused.  Run on the smallest configurations so that the test takes seconds."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                         text=True, timeout=280)
    return res.returncode, res.stdout, res.stderr


@pytest.mark.parametrize("workload", ["c1", "c2_causal"])
def test_bench_line(workload):
    rc, out, err = _bench("--workload", workload, "--steps", "5", "--warmup", "2", "--no-all-configs", "--no-mfma-probe")
    assert rc == 0, err[-2000:]
    lines = [l for l in out.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "parity"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "TFLOP/s" and d["data"] == "synthetic"
    assert d["vs_baseline"] is None and d["higher_is_better"] is True
    assert workload.split("_")[0] in d["config"]["workload"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["peak"] == 2500.0 and r["unit"] == "TFLOP/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and 0.0 < r["frac"] < 1.0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and "heads" in c["sample"]
    p = d["parity"]
    assert p["ok"] is True and p["all_outputs_finite"] is True
    assert p["o_max_abs"] <= 2e-2 and p["o_mean_abs"] <= 2e-3 and p["lse_max_abs"] <= 1e-2
    assert abs(d["value"] - d["config"]["flops_per_step"] / (d["ms_per_step"] * 1e-3) * 1e-12) < 1e-6 * max(1.0, d["value"])


def test_more_than_one_gpu_is_refused():
    rc, out, err = _bench("--gpus", "2")
    assert rc != 0 and out.strip() == "" and "ONE GPU" in err
