"""What can be checked of bench.py without a GPU: more than one GPU is refused with a message, before anything
touches a device."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    for extra_env, args in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ)
        env.update(extra_env)
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, env=env, timeout=120)
        assert r.returncode == 2
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


import pytest


@pytest.mark.gpu
def test_bench_line_carries_the_contract():
    """One JSON line on stdout with the keys the driver reads, the roofline object with its three fractions and the
    oracle timed beside it (a small workload, two steps: the contract, not the numbers)."""
    import json
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "cfg2", "--steps", "2", "--warmup", "1"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["unit"] == "GB/s" and d["vs_baseline"] is None
    assert d["data"] == "synthetic" and d["dtype"] == "i32" and "workload" in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert rf["frac"] == pytest.approx(rf["achieved"] / rf["peak"], abs=1e-3)
    assert rf["achieved"] == pytest.approx(d["config"]["bytes_min"] / (d["ms_per_step"] * 1e-3) / 1e9, rel=1e-3)
    assert 0 < rf["compulsory_frac"] < rf["frac"] and rf["compulsory_bytes"] < rf["algorithmic_bytes_per_launch"]
    assert (rf["traffic"] is None) == (rf["traffic_frac"] is None) == (rf["traffic_source"] is None)
    if rf["traffic"] is not None:                          # from the committed profile of this workload and launch shape
        assert rf["traffic_source"].startswith("profiles/") and rf["compulsory_bytes"] <= rf["traffic"]
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "GB/s" and 1 <= cb["cores"] <= cb["nproc"] and cb["value"] > 0
    assert d["parity_full_buffers_bitwise"] is True
