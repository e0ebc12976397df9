"""The benchmark's command line and output line."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_all_cores_baseline_slices_give_the_whole_tensors_result(oracle):
    """The all-cores leg of cpu_baseline steps contiguous ranges of blocks on separate threads: the
    result must be the whole tensor's, bit for bit (blocks are independent)."""
    import numpy as np
    sys.path.insert(0, ROOT)
    import bench
    n, K = 5 * 2048 + 777, 128
    assert bench.block_slices(n, K, 4) == [(0, 2816), (2816, 5632), (5632, 8448), (8448, n)]
    assert bench.block_slices(100, 128, 16) == [(0, 100)]
    rng = np.random.default_rng(5)
    th = (rng.standard_normal(n) * 0.02).astype(np.float32)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    whole, st_w = th.copy(), oracle.State.zeros(n, K, 5, 4)
    parts, st_p = th.copy(), oracle.State.zeros(n, K, 5, 4)
    for t in (1, 2, 3):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        oracle.step(whole, g, st_w, **hp, t=t)
        for lo, hi in bench.block_slices(n, K, 5):
            oracle.step(parts[lo:hi], g[lo:hi], bench.state_slice(oracle, st_p, lo, hi), **hp, t=t)
    assert np.array_equal(whole.view(np.uint32), parts.view(np.uint32))
    for a in ("um", "cv", "sm", "sv"):
        assert np.array_equal(getattr(st_w, a), getattr(st_p, a)), a


@pytest.mark.gpu
def test_output_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "adam-1tensor", "--steps", "5",
                        "--warmup", "2"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["unit"] == "params/s" and d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["dtype"] == "f32" and d["config"]["workload"] == "adam-1tensor" and "model" not in d["config"]
    assert abs(d["value"] - d["config"]["params"] / (d["ms_per_step"] * 1e-3)) <= 1e-6 * d["value"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12 and "traffic" in rf
    assert abs(rf["achieved"] - rf["algorithmic_bytes_per_launch"] / (rf["kernel_ms_avg"] * 1e-3) / 1e9) <= 1e-6 * rf["achieved"]
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "params/s" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    assert cb["one_thread_value"] > 0 and cb["os_cpu_count"] >= cb["cores"] and "cpu_model" in cb
    assert len(rf["kernel_source_sha256"]) == 16
