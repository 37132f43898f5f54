"""Turn rocprofv3 output of bench.py runs into the short summaries under profiles/.

`python bench.py --summarise DIR` (or `python bench_summarise.py DIR`) expects, under DIR, what
these three commands leave behind (run from the repository root on the MI355X machine after
`cd /tmp && export TMPDIR=/tmp && cd -`; ARGS = the bench.py arguments of the workload, e.g.
nothing for the headline, `--config 2 --layer 0`, `--block 60m`):

    rocprofv3 --kernel-trace --stats --output-format csv -d DIR/trace -o bench -- python3 bench.py ARGS --steps 200 --warmup 50 --no-cpu-baseline --no-extras > DIR/trace.log
    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR/fetch -o bench -- python3 bench.py ARGS --steps 10 --warmup 2 --settle-launches 20 --no-cpu-baseline --no-extras > DIR/fetch.log
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d DIR/write -o bench -- python3 bench.py ARGS --steps 10 --warmup 2 --settle-launches 20 --no-cpu-baseline --no-extras > DIR/write.log

(the counter passes are optional).  It writes profiles/bench_<key>_kernel_trace.md,
profiles/bench_<key>_hbm_traffic.md and the workload's entry of profiles/gemm_traffic.json, which
bench.py quotes as `roofline.traffic`.  <key> is the `config.key` of bench.py's own line.

Calibration of the byte counters: bench.py copies X once with a plain device-to-device copy of
known size; the counter values of that dispatch give the bytes one counter unit stands for.
"""
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
PROFILES = os.path.join(ROOT, "profiles")


def short(name):
    name = name.replace("grass::(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0][:80]


def find_csv(folder, suffix):
    hits = sorted(glob.glob(os.path.join(folder, "**", "*" + suffix), recursive=True))
    return hits[0] if hits else None


def bench_line(path):
    lines = [l for l in open(path).read().splitlines() if l.startswith("{")]
    return json.loads(lines[-1])


def counter_values(path, name):
    agg = collections.defaultdict(list)
    for row in csv.DictReader(open(path)):
        # kernels of this library (their full names carry its namespace) and the calibration copy
        if row["Counter_Name"] == name and (is_ours(row["Kernel_Name"]) or "copyBuffer" in row["Kernel_Name"]):
            agg[short(row["Kernel_Name"])].append(float(row["Counter_Value"]))
    return agg


def is_ours(name):
    return "grass" in name or "tn_gemm" in name or "pack_" in name or "adam" in name


def kernel_trace(folder, line, key, argv):
    stats = find_csv(os.path.join(folder, "trace"), "kernel_stats.csv")
    rows = list(csv.DictReader(open(stats)))
    out = [f"# rocprofv3 kernel trace: bench.py {argv}".rstrip(), "",
           f"Workload: {line['config']['workload']}", "",
           "Command (from the repository root on the MI355X box, after `cd /tmp && export TMPDIR=/tmp && cd -`):", "",
           f"    rocprofv3 --kernel-trace --stats --output-format csv -d DIR/trace -o bench -- python3 bench.py {argv} --steps {line['steps']} --warmup {line['warmup']} --no-cpu-baseline --no-extras".replace("  ", " "),
           "", "bench.py's own line from that run (HIP-event timing inside the profiled process):", ""]
    roof = line.get("roofline") or {}
    facts = [f"value = {line['value']:.1f} {line['unit']}", f"ms_per_step = {line['ms_per_step']:.4f}"]
    if "regular_step_ms" in line:
        facts.append(f"regular step = {line['regular_step_ms']:.4f} ms")
    if roof:
        facts.append(f"roofline: {roof['bound']}, {roof['achieved']:.1f} {roof['unit']} = {roof['frac']:.3f} of "
                     f"{roof['peak']:.0f} (avg launch {roof['avg_launch_ms']:.4f} ms)")
    if "step_tail" in line:
        t = line["step_tail"]
        facts.append(f"step tail by bench.py's stamped events = {t['ms'] * 1e3:.1f} us (under the profiler these "
                     "read a few us more than the profiler's own kernel times below; without it they agree)")
    if "settle_launches" in line:
        facts.append(f"settle phase: {line['settle_launches']} launches, GEMM {line['settle_gemm_ms_first_batch']:.4f} -> "
                     f"{line['settle_gemm_ms_last_batch']:.4f} ms")
    out += ["    " + "; ".join(facts), "",
            "Kernel statistics (kernels of this library; warm-up, settle phase and timed steps, refreshes included):", "",
            "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---:|---:|---:|---:|---:|"]
    for r in rows:
        if is_ours(r["Name"]):
            out.append("| %s | %s | %.2f | %.2f | %.2f | %.2f |" % (
                short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
                float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
    path = os.path.join(PROFILES, f"bench_{key}_kernel_trace.md")
    open(path, "w").write("\n".join(out) + "\n")
    return path


def algorithmic_mb(kernel, c, slices):
    """Read / written MB a kernel of the regular step has to move for the workload `c`."""
    T, m, n, r = c["T"], c["m"], c["n"], c["r"]
    if "tn_gemm_bf16" in kernel and "<true" not in kernel.split("tn_gemm_bf16")[1][:30]:
        return "%.0f / %.0f" % (2 * T * (r + n) / 1e6, slices * r * n * 4 / 1e6)
    if kernel.startswith("tn_gemm_gather_narrow"):  # the gather inside the GEMM: dY and X in, partial tiles out
        return "%.0f / %.0f" % (2 * T * (m + n) / 1e6, slices * r * n * 4 / 1e6)
    if kernel.startswith("pack_txm"):
        return "%.0f / %.0f" % (2 * T * m / 1e6, 2 * T * r / 1e6)
    if kernel.startswith("reduce_adam_scatter"):
        return "%.0f / %.0f" % ((slices * r * n * 4 + r * n * 10) / 1e6, r * n * 10 / 1e6)
    if kernel.startswith("adam_scatter"):
        return "%.0f / %.0f" % (r * n * 14 / 1e6, r * n * 10 / 1e6)
    if kernel.startswith("row_stats"):
        return "%.0f / %.0f" % (m * n * 4 / 1e6, m * 4 / 1e6)
    if kernel.startswith("gather_rows"):
        return "%.0f / %.0f" % (r * n * 4 / 1e6, r * n * 4 / 1e6)
    if "tn_gemm_bf16" in kernel:  # the full-gradient product of a refresh step
        return "%.0f / %.0f" % (2 * T * (m + n) / 1e6, m * n * 4 / 1e6)
    if kernel.startswith("align_rows"):
        return "%.0f / %.0f" % (2 * T * n / 1e6, 2 * T * ((n + 7) // 8 * 8) / 1e6)
    return ""


def hbm_traffic(folder, line, key, argv):
    fetch = find_csv(os.path.join(folder, "fetch"), "counter_collection.csv")
    write = find_csv(os.path.join(folder, "write"), "counter_collection.csv")
    if not fetch or not write:
        return None
    f, w = counter_values(fetch, "FETCH_SIZE"), counter_values(write, "WRITE_SIZE")
    c = line["config"]
    if "n" not in c:  # a block run: several layers, no single calibration size
        return None
    esz = 2 if line["dtype"] == "bf16" else 4
    copy_bytes = c["T"] * c["n"] * esz
    fc = max(v for k, vals in f.items() if "copyBuffer" in k for v in vals)
    wc = max(v for k, vals in w.items() if "copyBuffer" in k for v in vals)
    fu, wu = copy_bytes / fc, copy_bytes / wc
    slices = (line.get("step_tail") or {}).get("k_slices", 1)
    out = [f"# HBM traffic of the kernels of bench.py {argv} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)".replace("  ", " "), "",
           f"Workload: {c['workload']}", "", "Commands (two runs, one counter each):", "",
           f"    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR/fetch -o bench -- python3 bench.py {argv} --steps 10 --warmup 2 --settle-launches 20 --no-cpu-baseline --no-extras".replace("  ", " "),
           f"    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d DIR/write -o bench -- python3 bench.py {argv} --steps 10 --warmup 2 --settle-launches 20 --no-cpu-baseline --no-extras".replace("  ", " "),
           "",
           f"Calibration: bench.py copies X ({copy_bytes} bytes) once with a plain device-to-device copy "
           f"(`__amd_rocclr_copyBuffer`).  That dispatch reads FETCH_SIZE = {fc:.1f} and WRITE_SIZE = {wc:.1f}, so one "
           f"FETCH_SIZE unit stands for {fu:.1f} bytes and one WRITE_SIZE unit for {wu:.1f} bytes here; every figure "
           "below is the counter times that factor.", "",
           "| kernel | dispatches | FETCH_SIZE avg | read MB | WRITE_SIZE avg | written MB | algorithmic MB (read / written) |",
           "|---|---:|---:|---:|---:|---:|---|"]
    per_kernel = {}
    for k in sorted(f):
        if "copyBuffer" in k:
            continue
        fv, wv = f[k], w.get(k, [0.0])
        favg, wavg = sum(fv) / len(fv), sum(wv) / len(wv)
        per_kernel[k] = (len(fv), favg * fu, wavg * wu)
        out.append("| %s | %d | %.1f | %.1f | %.1f | %.1f | %s |" % (
            k, len(fv), favg, favg * fu / 1e6, wavg, wavg * wu / 1e6, algorithmic_mb(k, c, slices)))
    roof = line.get("roofline") or {}
    rec = None
    if roof.get("bound") == "mfma":
        hits = [v for k, v in per_kernel.items() if "tn_gemm_bf16_direct_kernel<false, false" in k]
        if hits:
            _, rd, wr = hits[0]
            rec = {"bytes_per_launch": rd + wr, "read_bytes": rd, "written_bytes": wr,
                   "what": "the compressed-gradient GEMM kernel"}
    elif roof.get("bound") == "hbm":
        # the whole regular step: every kernel of it, weighted by its launches per step
        tails = [v[0] for k, v in per_kernel.items() if k.startswith("reduce_adam_scatter")]
        steps = max(tails) if tails else 0
        step_kernels = ("pack_", "align_rows", "tn_gemm_bf16", "tn_gemm_gather_narrow", "reduce_adam_scatter",
                        "scatter_cols")
        rd = wr = 0.0
        for k, (calls, r_b, w_b) in per_kernel.items():
            if steps and k.startswith(step_kernels) and "<true" not in k[:40]:
                rd += r_b * calls / steps
                wr += w_b * calls / steps
        if steps:
            rec = {"bytes_per_launch": rd + wr, "read_bytes": rd, "written_bytes": wr,
                   "what": "all kernels of one regular step (gather, GEMM, fused tail)"}
            out += ["", "One regular step (its kernels weighted by launches per step): read %.1f MB, written %.1f MB; "
                    "algorithmic %.1f MB." % (rd / 1e6, wr / 1e6, roof["bytes_per_launch"] / 1e6)]
    path = os.path.join(PROFILES, f"bench_{key}_hbm_traffic.md")
    open(path, "w").write("\n".join(out) + "\n")
    if rec:
        rec.update({"source": os.path.relpath(path, ROOT), "fetch_unit_bytes": fu, "write_unit_bytes": wu})
        jpath = os.path.join(PROFILES, "gemm_traffic.json")
        table = json.load(open(jpath)) if os.path.exists(jpath) else {}
        table[f"{c['key']}:T={c['T']}"] = rec
        json.dump(table, open(jpath, "w"), indent=1)
    return path


def main(folder):
    line = bench_line(os.path.join(folder, "trace.log"))
    key = line["config"]["key"]
    argv = line["config"].get("argv", "")
    for flag in ("--no-cpu-baseline", "--no-extras"):
        argv = argv.replace(flag, "")
    import re
    argv = re.sub(r"--(steps|warmup|settle-launches)\s+\d+", "", argv)
    argv = " ".join(argv.split())
    print(kernel_trace(folder, line, key, argv))
    fline = line
    if os.path.exists(os.path.join(folder, "fetch.log")):
        fline = bench_line(os.path.join(folder, "fetch.log"))
        fline["roofline"] = line.get("roofline")  # timing from the trace run, counters from the counter runs
    print(hbm_traffic(folder, fline, key, argv))


if __name__ == "__main__":
    main(sys.argv[1])
