"""bench.py's one-line JSON contract, on a shortened token batch (runs in seconds)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                       capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, "exactly one JSON line"
    return json.loads(lines[0])


def test_layer_bench_line_has_every_field_of_the_contract():
    d = run_bench("--tokens", "4096", "--steps", "5", "--warmup", "2", "--cpu-seconds", "1")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config", "roofline",
                "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2
    assert d["higher_is_better"] is True and d["vs_baseline"] is None
    assert d["unit"] == "layer-steps/s" and d["dtype"] == "bf16" and d["data"] == "synthetic"
    assert abs(d["value"] * d["ms_per_step"] * 1e-3 - 1.0) < 1e-6
    assert "workload" in d["config"] and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    assert abs(r["achieved"] - r["flops_per_launch"] / (r["avg_launch_ms"] * 1e-3) / 1e12) < 1e-6 * r["achieved"]
    assert "traffic" in r and "traffic_source" in r  # measured bytes exist for the full-size workload only
    assert 10 <= d["settle_launches"] <= 400 and d["settle_gemm_ms_last_batch"] > 0
    t = d["step_tail"]
    assert t["ms"] > 0 and abs(t["GBs"] - t["algorithmic_bytes"] / (t["ms"] * 1e-3) / 1e9) < 1e-6 * t["GBs"]
    assert d["regular_step_ms"] > 0
    # the refresh step (one full-gradient product at 4x the flops) is the first timed step
    assert d["refresh_step_ms"] > d["regular_step_ms"] and "kept" in d["refresh_step"]
    assert d["detail"]["refresh_step_one_product_ms"] < d["detail"]["refresh_step_two_products_ms"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == d["unit"] and c["cores"] >= 1 and c["value"] > 0
    assert isinstance(c["sample"], str) and c["sample"]


def test_layer_bench_line_of_a_memory_bound_configuration():
    """The narrow layers of the small models are priced against HBM: the whole regular step."""
    d = run_bench("--config", "2", "--layer", "0", "--tokens", "8192", "--steps", "5", "--warmup", "2",
                  "--no-cpu-baseline", "--no-extras")
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    assert abs(r["achieved"] - r["bytes_per_launch"] / (r["avg_launch_ms"] * 1e-3) / 1e9) < 1e-6 * r["achieved"]
    assert r["bytes_per_launch"] == 2 * 8192 * (512 + 512) + 128 * 512 * 20
    assert d["step_tail"]["k_slices"] > 8 and d["config"]["key"] == "c2_attn_qkvo"


def test_layer_bench_with_the_two_product_refresh_step():
    d = run_bench("--tokens", "4096", "--steps", "3", "--warmup", "1", "--refresh", "two-products",
                  "--no-cpu-baseline", "--no-extras")
    assert d["refresh_step_ms"] > d["regular_step_ms"] and "not stored" in d["refresh_step"]


def test_layer_bench_of_a_single_step_still_prices_the_gemm():
    """One timed step is the refresh step (no compressed-gradient product in it): the GEMM and the
    tail are then timed on regular steps after the timed region."""
    d = run_bench("--tokens", "4096", "--steps", "1", "--warmup", "1", "--no-cpu-baseline", "--no-extras")
    assert d["steps"] == 1 and abs(d["refresh_step_ms"] - d["ms_per_step"]) < 0.05 * d["ms_per_step"]
    assert d["roofline"]["avg_launch_ms"] > 0 and d["step_tail"]["ms"] > 0


def test_adam_cold_mode_prints_its_two_rates():
    d = run_bench("--adam-cold", "--config", "2", "--layer", "0")
    for key in ("adam_scatter_cold", "plain_add_cold_same_elements"):
        assert d[key]["launches"] == 200 and d[key]["GBs"] > 0
    assert d["adam_scatter_cold"]["bytes"] == 128 * 512 * 24


def test_block_bench_line():
    d = run_bench("--block", "60m", "--tokens", "2048", "--steps", "4", "--warmup", "1")
    assert d["unit"] == "block-steps/s" and d["n_gpus"] == 1 and d["value"] > 0
    assert "workload" in d["config"]
