"""bench.py's contract with whoever runs it: what it refuses, that the traffic figure it prints was
measured on the kernel source as it stands, and (on the GPU) the shape of its one JSON line."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figure_was_measured_on_the_present_kernel_source():
    """roofline.traffic is a counter reading taken in a profiler run, stored as a constant beside the
    SHA-1 of the kernel source it was taken on.  A change to that source without a new counter pass
    fails here (and bench.py then prints traffic_stale: true)."""
    sys.path.insert(0, ROOT)
    import bench
    assert bench.ATTN_TRAFFIC_MEASURED_ON_SHA1 == bench.kernel_source_sha1(), \
        "the attention kernel's source changed after its HBM traffic was measured: run the FETCH_SIZE / WRITE_SIZE " \
        "passes again (profiles/attn_layer7b_step32_6580cached_204new.txt names the commands) and update both constants"


@pytest.mark.gpu
def test_json_line_of_a_short_run():
    r = subprocess.run([sys.executable, BENCH, "--steps", "20", "--warmup", "5", "--no-latency", "--no-extra",
                        "--cpu-seconds", "1"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    d = json.loads(lines[0])
    for key, kind in (("metric", str), ("value", float), ("unit", str), ("n_gpus", int), ("steps", int), ("warmup", int),
                      ("ms_per_step", float), ("higher_is_better", bool), ("scaling", str), ("dtype", str),
                      ("data", str), ("config", dict), ("roofline", dict), ("cpu_baseline", dict)):
        assert isinstance(d[key], kind), key
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 5 and d["vs_baseline"] is None
    assert d["unit"] == "tokens/s" and d["dtype"] == "bf16" and d["data"] == "synthetic" and d["higher_is_better"]
    assert "workload" in d["config"] and "model" not in d["config"]
    # value and ms_per_step describe the same timed region: 204 new tokens per step
    assert abs(d["value"] - 204 / (d["ms_per_step"] * 1e-3)) <= 1e-3 * d["value"]
    assert 0.02 < d["ms_per_step"] < 0.2
    ro = d["roofline"]
    assert ro["bound"] == "mfma" and ro["unit"] == "TFLOP/s" and ro["peak"] == 2500.0
    assert abs(ro["frac"] - ro["achieved"] / ro["peak"]) < 1e-3
    # achieved = the launch's algorithmic flops over the kernel's own average duration
    assert abs(ro["achieved"] - ro["flops_per_launch"] / (ro["avg_launch_us"] * 1e-6) / 1e12) < 0.5
    assert ro["avg_launch_us"] * 1e-3 < d["ms_per_step"], "the kernel is part of the step"
    assert ro["traffic"] > ro["algorithmic_bytes_per_launch"] > 0 and ro["traffic_stale"] is False
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "tokens/s" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    assert d["value"] > 100 * cb["value"]
    legs = d["rope_append"]["legs"]
    assert [leg["n_new"] for leg in legs] == [204, 3520] and all(0 < leg["frac_of_hbm_peak"] < 1 for leg in legs)
