"""bench_summarise.py on a small synthetic rocprofv3 output folder (CPU only): the kernel-trace
table, the byte calibration against the known-size copy, and the traffic record bench.py quotes."""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench_summarise  # noqa: E402

GEMM = ("void grass::(anonymous namespace)::tn_gemm_bf16_direct_kernel<false, false, false, false>"
        "(grass::(anonymous namespace)::GemmArgs)")
TAIL = ("void grass::(anonymous namespace)::reduce_adam_scatter_few_kernel<unsigned short, float, false>"
        "(grass::TailSets, int, long, long, long, grass::(anonymous namespace)::AdamParams, float)")
COPY = "__amd_rocclr_copyBuffer"


def counter_csv(path, name, rows):
    with open(path, "w") as f:
        f.write('"Kernel_Name","Counter_Name","Counter_Value"\n')
        for kernel, value in rows:
            f.write(f'"{kernel}","{name}",{value}\n')


def test_summaries_and_traffic_record(tmp_path, monkeypatch):
    T, m, n, r = 4096, 512, 512, 128
    line = {"metric": "m", "value": 1000.0, "unit": "layer-steps/s", "steps": 200, "warmup": 50,
            "ms_per_step": 1.0, "dtype": "bf16", "regular_step_ms": 0.99,
            "config": {"workload": "synthetic", "m": m, "n": n, "T": T, "r": r, "layer": "x", "key": "unit_test",
                       "argv": "--config 2 --steps 200 --warmup 50 --no-extras"},
            "roofline": {"bound": "mfma", "achieved": 1400.0, "peak": 2500.0, "unit": "TFLOP/s", "frac": 0.56,
                         "avg_launch_ms": 0.77},
            "step_tail": {"ms": 0.027, "GBs": 5500.0, "k_slices": 4}}
    d = tmp_path / "prof"
    for sub in ("trace", "fetch", "write"):
        (d / sub).mkdir(parents=True)
    (d / "trace.log").write_text("noise\n" + json.dumps(line) + "\n")
    (d / "fetch.log").write_text(json.dumps(line) + "\n")
    (d / "trace" / "bench_kernel_stats.csv").write_text(
        '"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
        f'"{GEMM}",250,192500000,770000.0,73.0,745000,880000,1.0\n'
        f'"{TAIL}",250,6750000,27000.0,2.6,25000,31000,1.0\n'
        '"void at::native::something<float>(int)",5,100,20.0,0.1,10,30,1.0\n')
    copy_bytes = T * n * 2
    # the copy of known size reads copy_bytes / 2048 fetch units and writes copy_bytes / 1024 write units
    counter_csv(d / "fetch" / "bench_counter_collection.csv", "FETCH_SIZE",
                [(COPY, copy_bytes / 2048), (COPY, 3.0), (GEMM, 1000.0), (GEMM, 3000.0), (TAIL, 50.0)])
    counter_csv(d / "write" / "bench_counter_collection.csv", "WRITE_SIZE",
                [(COPY, copy_bytes / 1024), (GEMM, 500.0), (GEMM, 500.0), (TAIL, 40.0)])
    out = tmp_path / "profiles"
    out.mkdir()
    monkeypatch.setattr(bench_summarise, "PROFILES", str(out))
    monkeypatch.setattr(bench_summarise, "ROOT", str(tmp_path))
    bench_summarise.main(str(d))
    trace = (out / "bench_unit_test_kernel_trace.md").read_text()
    assert "tn_gemm_bf16_direct_kernel<false, false, false, false> | 250 | 770.00" in trace
    assert "at::native" not in trace  # kernels of the library only
    assert "bench.py --config 2 --steps 200 --warmup 50 --no-cpu-baseline --no-extras" in trace
    traffic = (out / "bench_unit_test_hbm_traffic.md").read_text()
    assert "2048.0 bytes" in traffic and "1024.0 bytes" in traffic  # the calibration
    rec = json.load(open(out / "gemm_traffic.json"))["unit_test:T=4096"]
    assert rec["read_bytes"] == 2000.0 * 2048 and rec["written_bytes"] == 500.0 * 1024
    assert rec["bytes_per_launch"] == rec["read_bytes"] + rec["written_bytes"]
    assert rec["source"].endswith("bench_unit_test_hbm_traffic.md")
