"""The benchmark's command-line contract, as far as it can be checked without a GPU, and its JSON line on one."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one-GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""  # no JSON line that could be mistaken for a result


def test_workload_recipes_are_deterministic_and_sized_as_named():
    sys.path.insert(0, ROOT)
    import numpy as np

    import fls_workloads as wl

    cfg = wl.CONFIGS["C1"]
    W1, X1 = wl.make_inputs(cfg)
    W2, X2 = wl.make_inputs(cfg)
    assert np.array_equal(W1, W2) and np.array_equal(X1, X2)
    assert W1.shape == (1024, 1024) and X1.shape == (8, 1024) and W1.dtype == np.uint16
    assert abs(np.count_nonzero(W1) / W1.size - 0.2) < 0.01
    c2 = wl.CONFIGS["C2"]
    assert (c2.M, c2.K, c2.N, c2.beta, c2.mask) == (28672, 7168, 16, 0.8, "magnitude")
    layer = wl.decoder_layer(7168, 28672, 16, 0.8)
    assert [(c.M, c.K) for c in layer] == [(21504, 7168), (7168, 7168), (28672, 7168), (7168, 28672)]
    assert len({c.seed for c in layer}) == 4


@pytest.mark.gpu
def test_bench_line_carries_the_contract_fields():
    """A short run of the small configuration: one JSON line with the fields the driver reads."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "C1", "--steps", "50", "--warmup", "5"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 50 and out["warmup"] == 5 and out["dtype"] == "f16"
    assert out["vs_baseline"] is None and out["data"] == "synthetic" and "workload" in out["config"]
    roof = out["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert roof["traffic"] is None  # nobody measured C1's HBM traffic: the line must not pretend
    ceil = out["stream_ceiling"]
    assert ceil["GBps"] > 0 and ceil["bytes"] == out["config"]["blob_bytes"]
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    assert out["parity"]["max_rel_err_vs_oracle"] <= out["parity"]["tolerance"] and out["parity"]["rows_checked"] == 1024
