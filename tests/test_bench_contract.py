"""bench.py's command-line contract: one JSON line with the agreed keys; more than one GPU is refused."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "1", "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "ceilings", "configs"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 3 and out["warmup"] == 1
    assert out["unit"] == "TFLOP/s" and out["higher_is_better"] is True and out["data"] == "synthetic"
    assert out["vs_baseline"] is None and out["dtype"] == "fp8"
    assert "workload" in out["config"] and "model" not in out["config"]
    assert out["value"] > 0 and out["ms_per_step"] > 0
    roof = out["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    # config 1 has 24 rows per expert: its GEMMs stream weights, so the bound is HBM; the full-size configs in
    # `configs` carry their own bound
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert set(out["configs"]) == {"cfg2", "cfg3"}
    for c in out["configs"].values():
        assert c["ms_per_step"] > 0 and c["roofline"]["bound"] in ("hbm", "mfma") and 0 < c["roofline"]["frac"] < 1
    ceil = out["ceilings"]
    assert 1000 < ceil["copy_GBs"] < 8000
    assert 1000 < ceil["fp8_mfma_loop_with_block_scaling_tflops"] <= ceil["fp8_mfma_loop_tflops"] * 1.05 < 5250
    cpu = out["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1
