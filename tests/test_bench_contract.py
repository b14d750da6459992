"""The benchmark's command-line contract and its CPU leg (no GPU needed for the first two)."""
import json
import os
import subprocess
import sys

import pytest

from datagen import configs as cf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and not res.stdout.strip()


def test_cpu_baseline_leg_on_the_toy_workload():
    sys.path.insert(0, ROOT)
    import bench
    w = cf.WORKLOADS["toy"]
    out = bench.cpu_baseline(w["model"], w["src"], w["dst"], 0, cf.seed_of("toy"), target_seconds=0.2)
    assert out["kind"] == "oracle" and out["unit"] == "GB/s" and out["cores"] >= 1
    assert out["value"] > 0 and out["value_one_core"] > 0 and "destination buffers of rank 0" in out["sample"]


def test_source_fingerprint_follows_the_kernel_sources(tmp_path):
    sys.path.insert(0, ROOT)
    import bench
    fp = bench.kernel_sources_fingerprint()
    assert len(fp) == 16 and fp == bench.kernel_sources_fingerprint()
    stored = [ln.split("=")[1].strip() for ln in open(os.path.join(ROOT, "profiles", "k_copy_tiles_gqa70b_rank11_hbm_traffic.txt"))
              if ln.startswith("kernel_sources_fingerprint")]
    assert len(stored) == 1 and len(stored[0]) == 16   # (equal to fp only while the profile is current)


@pytest.mark.gpu
def test_json_line_has_the_contract_fields():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--headline-only", "--no-cpu-baseline", "--steps", "3", "--warmup", "1"],
                         capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [ln for ln in res.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
              "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["config"]["workload"] == "gqa70b rank 11" and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and 0.5 < r["frac"] < 1.0
    assert d["value"] <= r["achieved"] * 1.001           # the whole step cannot beat its copy kernel
    assert abs(d["value"] - d["bytes"]["moved_read_plus_write"] / (d["ms_per_step"] * 1e-3) / 1e9) < 1e-6 * d["value"]
    for k in ("plain_copy_gbps", "read_only_gbps", "write_only_gbps", "read_write_harmonic_gbps", "traffic", "traffic_source"):
        assert k in r, k
    assert (r["traffic"] is None) == (not str(r["traffic_source"]).startswith("stored profile figure"))
