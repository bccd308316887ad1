"""bench.py's command line and output: one JSON line with the fields its readers rely on.  The multi-GPU refusal is
checked without a GPU; the run itself needs one (a child process, a few timed steps)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


@pytest.mark.gpu
@pytest.mark.usefixtures("built_library")
def test_one_json_line_with_roofline_and_cpu_baseline():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and "workload" in d["config"]
    r = d["roofline"]
    assert r["bound"] in ("hbm", "mfma", "alu", "lds") and r["unit"] in ("GB/s", "TFLOP/s")
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and 0 < r["frac"] < 1
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and "sample" in cb
    # the GPU path does at least a thousand times the single-core oracle's move evaluations per second
    assert d["value"] > 1000 * cb["value"]
    # the step's move count and winner are the workload's, fixed by its seed; the oracle says what they are
    import numpy as np

    import oracle
    from gen import WORKLOADS, make_matrix
    w = WORKLOADS[2]
    costs, _, moves = oracle.restarts(make_matrix(2), oracle.SUM, w.search_seed, 0, w.restarts)
    assert d["move_evals_per_step"] == int(((moves.astype(np.int64) + 1) * oracle.neighbourhood_size(w.n, oracle.SUM)).sum())
    assert d["best_cost"] == int(costs.min())
    # the directed max-hop search of the same step, and the other roofline entries
    w3 = WORKLOADS[3]
    costs3, _, moves3 = oracle.restarts(make_matrix(3), oracle.MAX_DIRECTED, w3.search_seed, 0, w3.restarts)
    assert d["move_evals_per_step_c3"] == int(((moves3.astype(np.int64) + 1)
                                               * oracle.neighbourhood_size(w3.n, oracle.MAX_DIRECTED)).sum())
    assert d["best_cost_c3"] == int(costs3.min())
    r3 = d["roofline_c3"]
    assert r3["bytes_per_move"] == 16 and abs(r3["frac"] - 2 * r3["frac_at_storage_width"]) < 1e-9
    rb = d["roofline_batch"]
    assert rb["bound"] == "hbm" and 0 < rb["frac_cold"] < 1 and rb["cold"]["batch"] == 1 << 22
    # `value` is the rate of the whole search call, so it cannot exceed the rate of its search kernel alone
    assert d["value"] <= d["move_evals_per_step"] / (r["kernel_ms"] * 1e-3) * 1.05
