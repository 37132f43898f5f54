#!/usr/bin/env python3
"""Benchmark of the GRASS layer step on one MI355X.

One "step" is one pass of Algorithm 1 for one linear layer over one synthetic token batch
that is already resident in HBM.  On steps with t = 0 (mod K, K = 200 as in the paper's
pretraining runs) it is the refresh step: the full gradient formed once and kept in fp32, its
row norms, the selection, the state reset, the selected rows of the kept gradient as G_C, Adam
and the scatter into W (--refresh two-products: row norms in the GEMM epilogue without storing
G, then a regular step).  On every other step: the compressed gradient, Adam on r x n, and the
scatter into W.  The timed region starts at t = 0, so it always contains exactly one refresh
step per 200 steps.

Prints ONE JSON line: metric, value (layer steps per second), ms_per_step, the workload, a
`roofline` object (for layers above the ridge the compressed-gradient GEMM against the matrix
cores, timed by events stamped with the kernel's own start and end; for the others the whole
regular step against HBM) and a `cpu_baseline` object (the fp64 oracle on the host cores, on a
bounded sample).  Only one GPU is supported.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2406_17660_amd import grass, workloads  # noqa: E402
from paper_2406_17660_amd.layer import AdamHyper, GrassLayer  # noqa: E402

PEAK_BF16_MFMA_TFLOPS = 2500.0  # MI355X dense bf16
PEAK_HBM_GBS = 8000.0
REFRESH_EVERY = 200  # the paper's K


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=50,
                   help="untimed steps first: the chip needs some tens of launches after an idle period to settle at its sustained clock")
    p.add_argument("--config", type=int, default=None,
                   help="workload configuration 1-5 (default: 5, or the one a --block belongs to)")
    p.add_argument("--layer", type=int, default=0, help="index into the config's layer list")
    p.add_argument("--tokens", type=int, default=None, help="override T (debug)")
    p.add_argument("--side", choices=["rows", "cols"], default="rows",
                   help="rows: select r rows of W (default); cols: right-hand projection, r columns")
    p.add_argument("--block", choices=sorted(workloads.BLOCKS), default=None,
                   help="time Algorithm 1 over all seven linear layers of one LLaMA block "
                        "(grouped q/k/v and gate/up calls) instead of the single layer")
    p.add_argument("--layout", choices=["txm", "mxt"], default="txm",
                   help="storage of dY: T x m (what the headline is quoted on) or m x T, whose "
                        "selected rows are contiguous and are gathered inside the GEMM")
    p.add_argument("--adam-state", choices=["f32", "bf16"], default="f32",
                   help="dtype of the Adam moments (the headline configuration keeps them in fp32)")
    p.add_argument("--graph", action="store_true",
                   help="with --block: capture the regular step into a HIP graph and replay it")
    p.add_argument("--concurrent-groups", action="store_true",
                   help="with --block: every group of layers on a HIP stream of its own")
    p.add_argument("--refresh", choices=["one-product", "two-products"], default="one-product",
                   help="refresh steps: the full gradient formed once and kept, its selected rows "
                        "being the step's compressed gradient (Algorithm 1 as printed), or the "
                        "statistic taken in the GEMM epilogue without storing G and the compressed "
                        "gradient recomputed as on a regular step")
    p.add_argument("--settle-launches", type=int, default=400,
                   help="cap of the untimed settle phase (steps run until the GEMM's time stops falling)")
    p.add_argument("--summarise", metavar="DIR", default=None,
                   help="no benchmark: turn the rocprofv3 output under DIR (see bench_summarise.py) "
                        "into the summaries under profiles/")
    p.add_argument("--clock-trace", action="store_true",
                   help="no benchmark line: sample the GPU clock (rocm-smi) while the 7B attention "
                        "layer's kernels and the matrix-core probes run back to back, and print a "
                        "markdown table (the evidence behind the power-bound reading of the GEMM)")
    p.add_argument("--adam-cold", action="store_true",
                   help="run nothing but grass_adam_scatter on state that is not in the caches (eight "
                        "sets of G_C, M, V, W cycled) and a plain a + b -> c stream of the same element "
                        "count, 200 launches each, and print one JSON line: the command behind "
                        "profiles/adam_scatter_cold_*.md")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-extras", action="store_true", help="skip the naive comparator etc.")
    p.add_argument("--cpu-seconds", type=float, default=15.0)
    return p.parse_args()


def ev():
    e = torch.cuda.Event(enable_timing=True)
    e.record()  # creates the handle so that the library can re-record it
    return e


def time_calls(fn, iters, warmup=2):
    """Median and minimum time of fn() in ms, measured with events on the current stream."""
    for _ in range(warmup):
        fn()
    pairs = []
    for _ in range(iters):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    ms = [a.elapsed_time(b) for a, b in pairs]
    return float(np.median(ms)), float(np.min(ms))


def cpu_baseline(cfg, layer, dY, X, state, W, seconds):
    """The fp64 oracle, untuned, on this machine's host cores: compressed gradient on a bounded
    sample of the selected rows (scaled to all r rows) plus Adam and scatter at full size."""
    from oracle import ref  # test infrastructure; used here only for the reported baseline

    def host(t):
        t = t.cpu()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    cores = len(os.sched_getaffinity(0))
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    dYh, Xh = host(dY), host(X)
    # the oracle's inputs are seeded draws of its own (nothing the GPU computed): r rows drawn
    # with replacement, unit scales, a normal compressed gradient for the Adam + update leg
    rng = np.random.default_rng(2406)
    r = state.r
    idx = np.sort(rng.integers(0, state.m, r)).astype(np.int32)
    rho = np.ones(r, np.float32)
    rows = min(r, cores)
    t0 = time.perf_counter()
    ref.compressed_grad(dYh, Xh, idx[:rows], rho[:rows])
    t_probe = time.perf_counter() - t0
    # grow the sample towards the time budget, in multiples of the core count
    want = int(seconds / max(t_probe, 1e-3)) * rows
    want = max(rows, min(r, want // cores * cores))
    if want > rows:
        rows = want
        t0 = time.perf_counter()
        ref.compressed_grad(dYh, Xh, idx[:rows], rho[:rows])
        t_probe = time.perf_counter() - t0
    t_cgrad_full = t_probe * r / rows
    GC = rng.standard_normal((r, state.n))
    M = np.zeros_like(GC)
    V = np.zeros_like(GC)
    Wd = W.cpu().to(torch.float64).numpy()
    a = state.adam
    t0 = time.perf_counter()
    U = ref.adam_rows(GC, M, V, a.lr, a.beta1, a.beta2, a.eps, 1)
    ref.scatter_update(Wd, idx, rho, state.alpha, U)
    t_tail = time.perf_counter() - t0
    step_s = t_cgrad_full + t_tail
    return {"value": 1.0 / step_s, "unit": "layer-steps/s", "cores": cores, "kind": "oracle",
            "sample": f"regular step: compressed_grad timed on {rows} of {r} selected rows "
                      f"(all n, all T; {t_probe:.1f} s) and scaled by {r / rows:.0f}, plus "
                      f"adam_rows + scatter_update at full size ({t_tail:.2f} s)"}


def measured_traffic(key, T):
    """(bytes, where from): HBM bytes per launch of the dominant kernel as measured with rocprofv3
    --pmc FETCH_SIZE / WRITE_SIZE in an earlier profiler run of this command (the counters cannot
    be read from inside the process).  profiles/gemm_traffic.json is written from such runs by
    `bench.py --summarise`; (None, None) if nothing is recorded for this workload."""
    path = os.path.join(ROOT, "profiles", "gemm_traffic.json")
    if not os.path.exists(path):
        return None, None
    rec = json.load(open(path)).get(f"{key}:T={T}")
    if not rec:
        return None, None
    return rec["bytes_per_launch"], (f"{rec['source']} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an "
                                     "earlier profiler run of this workload; not measured in this run)")


def settle(run_steps, cap):
    """Untimed steps until the chip has reached the clock it sustains under this load: after an
    idle period the first tens of GEMM launches run at a lower clock.  Steps are issued in
    batches of 10 with events around their GEMM kernels; the phase ends when a batch is no
    faster than the one before it (within 0.5 %) twice in a row, or at `cap` launches.
    Returns (launches, first batch's mean GEMM ms, last batch's)."""
    done, prev, first, calm = 0, None, None, 0
    while done < cap:
        events = [(ev(), ev()) for _ in range(10)]
        run_steps(10, events)
        torch.cuda.synchronize()
        cur = float(np.mean([a.elapsed_time(b) for a, b in events]))
        done += 10
        first = cur if first is None else first
        if prev is not None and cur >= prev * 0.995:
            calm += 1
            if calm == 2:
                break
        else:
            calm = 0
        prev = cur
    return done, first, prev if prev is not None else first


def layer_figures(cfg, layer, steps=40):
    """Regular-step figures of one more layer of the configuration (secondary measurements for
    the `detail` object): step time, the GEMM kernel's rate, the step's HBM rate, and the naive
    route (full gradient, then a row gather) beside the compressed gradient."""
    L = cfg.layers[layer]
    T, m, n, r = cfg.T, L.m, L.n, cfg.r
    dY = workloads.make_dY(cfg, layer, 0, "cuda")
    X = workloads.make_X(cfg, layer, 0, "cuda")
    W = workloads.make_W(cfg, layer, "cuda")
    st = GrassLayer(m, n, r, T, cfg.dtype, cfg.method, cfg.replacement, alpha=cfg.alpha,
                    adam=AdamHyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps), seed=workloads.BASE_SEED,
                    store_GC=False)
    st.refresh(dY, X, reset_state=True)
    for _ in range(10):
        st.step(dY, X, W)
    gemm_events = [(ev(), ev()) for _ in range(steps)]
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for t in range(steps):
        st.step(dY, X, W, gemm_events[t])
    b.record()
    torch.cuda.synchronize()
    step_ms = a.elapsed_time(b) / steps
    gemm_ms = float(np.mean([x.elapsed_time(y) for x, y in gemm_events]))
    flops = 2.0 * r * T * n
    esz = 2 if cfg.dtype == torch.bfloat16 else 4
    step_bytes = esz * T * (m + n) + r * n * (4 * st.M.element_size() + 2 * esz)
    call_ms, _ = time_calls(lambda: st.compressed_grad(dY, X), 10, warmup=2)
    dense_ms, _ = time_calls(lambda: st.full_gradient(dY, X), 3, warmup=1)
    tmp = torch.empty((r, n), dtype=torch.float32, device="cuda")
    gather_ms, _ = time_calls(lambda: grass.gather_rows(st.G, st.idx, st.rho, tmp), 10)
    tile, slices = grass.cgrad_plan(T, n, r, st.dt, m=m)
    return {"layer": L.name, "m": m, "n": n, "T": T, "r": r, "regular_step_ms": step_ms,
            "layer_steps_per_s": 1e3 / step_ms, "gemm_kernel_ms": gemm_ms,
            "gemm_kernel_tflops": flops / (gemm_ms * 1e-3) / 1e12,
            "gemm_kernel_frac_mfma": flops / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
            "step_algorithmic_GBs": step_bytes / (step_ms * 1e-3) / 1e9,
            "step_frac_hbm": step_bytes / (step_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "flop_per_input_byte": flops / (esz * T * (m + n)), "gemm_tile": tile, "k_slices": slices,
            "compressed_grad_call_ms": call_ms, "naive_full_grad_ms": dense_ms,
            "naive_gather_ms": gather_ms,
            "speedup_vs_naive_full_G_then_gather": (dense_ms + gather_ms) / call_ms}


def clock_trace(cfg):
    """What clock the chip sustains under each kind of load of the 7B attention layer step.
    rocm-smi is polled from a thread while each load runs back to back for about three seconds;
    prints a markdown table with the rate each load reached and the shader clocks seen."""
    import re
    import subprocess
    import threading
    from paper_2406_17660_amd import probe as mfma_probe

    dev = "cuda"
    L = cfg.layers[0]
    T, m, n, r = cfg.T, L.m, L.n, cfg.r
    dY = workloads.make_dY(cfg, 0, 0, dev)
    X = workloads.make_X(cfg, 0, 0, dev)
    W = workloads.make_W(cfg, 0, dev)
    adam = AdamHyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps)
    st = GrassLayer(m, n, r, T, cfg.dtype, cfg.method, cfg.replacement, alpha=cfg.alpha, adam=adam,
                    seed=workloads.BASE_SEED, store_GC=False)
    st.refresh(dY, X)
    dYt = dY.t().contiguous()
    st_t = GrassLayer(m, n, r, T, cfg.dtype, cfg.method, cfg.replacement, alpha=cfg.alpha, adam=adam,
                      seed=workloads.BASE_SEED, layout=grass.DY_MxT)
    st_t.idx.copy_(st.idx)
    st_t.rho.copy_(st.rho)
    g = torch.Generator(device=dev)
    g.manual_seed(workloads.BASE_SEED + 99)
    vals = torch.randn(32768, generator=g, device=dev)
    left = (torch.arange(32768, device=dev) // 2048) % 8 < 4
    vals = torch.where(left, vals * 0.1, vals).to(torch.bfloat16)

    samples, stop = [], [False]

    def sampler():
        while not stop[0]:
            t = time.time()
            try:
                o = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True,
                                   text=True, timeout=5).stdout
            except Exception as e:  # the read-out is best effort
                o = str(e)
            samples.append((t, o))

    def sclk_mhz(text):
        try:
            card = next(iter(json.loads(text).values()))
        except Exception:
            return None
        for k, v in card.items():
            if "sclk" in k.lower():
                hit = re.search(r"(\d+)\s*Mhz", str(v), flags=re.I)
                if hit:
                    return int(hit.group(1))
        return None

    flops = 2.0 * r * T * n
    rows = []

    def phase(name, fn, unit_of_work, seconds=3.0):
        torch.cuda.synchronize()
        t0, k = time.time(), 0
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        while time.time() - t0 < seconds:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()
            k += 20
        b.record()
        torch.cuda.synchronize()
        t1 = time.time()
        ms = a.elapsed_time(b) / k
        clocks = [c for c in (sclk_mhz(o) for t, o in samples if t0 + 0.5 <= t <= t1) if c]
        rows.append((name, ms, unit_of_work(ms), clocks))

    th = threading.Thread(target=sampler, daemon=True)
    th.start()
    try:
        time.sleep(2.5)
        idle = [c for c in (sclk_mhz(o) for _, o in samples) if c]
        rows.append(("idle", None, "", idle))
        st.GC.normal_()
        phase("Adam + row update alone (grass_adam_scatter, HBM-bound)", lambda: st.adam_scatter(W),
              lambda ms: "%.0f GB/s" % (24.0 * r * n / (ms * 1e-3) / 1e9))
        for name, source in (("matrix instruction only, constant operands", mfma_probe.CONSTANTS),
                             ("matrix instruction only, operands like the GEMM's inputs, in registers", mfma_probe.REGISTERS),
                             ("the same operands read from LDS fragment by fragment", mfma_probe.LDS)):
            out = torch.empty(256 * 256, dtype=torch.float32, device=dev)
            fl = [0.0]

            def one(source=source, out=out, fl=fl):
                import ctypes as C
                f = C.c_double(0.0)
                rc = mfma_probe.lib().mfma_rate_probe(
                    source, C.c_void_p(vals.data_ptr()), vals.numel() * 2, C.c_void_p(out.data_ptr()),
                    out.numel(), 2000, C.byref(f), C.c_void_p(torch.cuda.current_stream().cuda_stream))
                assert rc == 0
                fl[0] = f.value
            phase(name, one, lambda ms, fl=fl: "%.0f TFLOP/s" % (fl[0] / (ms * 1e-3) / 1e12))
        phase("compressed-gradient GEMM alone, dY stored m x T (row-gathering kernel, no gather pass)",
              lambda: st_t.compressed_grad(dYt, X), lambda ms: "%.0f TFLOP/s (whole call)" % (flops / (ms * 1e-3) / 1e12))
        phase("regular steps, dY stored T x m (gather 20 %, GEMM 75 %, fused tail 3 % of the time)",
              lambda: st.step(dY, X, W), lambda ms: "%.0f TFLOP/s over the whole step" % (flops / (ms * 1e-3) / 1e12))
    finally:
        stop[0] = True
        th.join(10)
    print("| load (about 3 s back to back) | ms per launch | rate | sclk samples | sclk MHz min / median / max |")
    print("|---|---:|---|---:|---|")
    for name, ms, rate, clocks in rows:
        c = ("%d / %d / %d" % (min(clocks), int(np.median(clocks)), max(clocks))) if clocks else "no read-out"
        print("| %s | %s | %s | %d | %s |" % (name, "" if ms is None else "%.4f" % ms, rate, len(clocks), c))


def bench_adam_cold(args, cfg):
    """grass_adam_scatter alone, cold: what a profiler needs to see that kernel by itself."""
    L = cfg.layers[args.layer]
    m, n, r = L.m, L.n, cfg.r
    dev = "cuda"
    g = torch.Generator(device=dev)
    g.manual_seed(workloads.BASE_SEED + 7)
    idx = torch.sort(torch.randint(0, m, (r,), generator=g, device=dev, dtype=torch.int32)).values
    rho = torch.ones(r, device=dev)
    sdt = torch.bfloat16 if args.adam_state == "bf16" else torch.float32
    sets = [(torch.randn((r, n), generator=g, device=dev), torch.zeros((r, n), dtype=sdt, device=dev),
             torch.zeros((r, n), dtype=sdt, device=dev), workloads.make_W(cfg, args.layer, dev))
            for _ in range(8)]
    trio = [tuple(torch.randn((r, n), generator=g, device=dev) for _ in range(3)) for _ in range(8)]
    esz = 2 if cfg.dtype == torch.bfloat16 else 4
    adam_bytes = r * n * (4 + 4 * sets[0][1].element_size() + 2 * esz)

    def adam(k):
        g_, m_, v_, w_ = sets[k % 8]
        grass.adam_scatter(g_, m_, v_, cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, 1 + k, w_, idx, rho, cfg.alpha)

    def add(k):
        x_, y_, z_ = trio[k % 8]
        torch.add(x_, y_, out=z_)

    out = {"workload": f"config {cfg.cid} layer {L.name}: r={r}, n={n}, W {m}x{n}, {args.adam_state} moments; "
                       "eight sets cycled (0.8 GB: nothing stays in the 256 MB last-level cache)"}
    for name, fn, nbytes in (("adam_scatter_cold", adam, adam_bytes), ("plain_add_cold_same_elements", add, 12 * r * n)):
        for k in range(16):
            fn(k)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for k in range(200):
            fn(k)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / 200  # back to back: includes the launch gaps
        out[name] = {"launches": 200, "ms_per_launch_back_to_back": ms, "bytes": nbytes,
                     "GBs": nbytes / (ms * 1e-3) / 1e9, "frac_hbm": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
    print(json.dumps(out))


def bench_block(args, cfg):
    """Amortised block steps/s: every layer of one block, refresh every 200 steps, the
    re-warm-up schedule supplying the learning rate.  A secondary measurement: the headline
    metric stays the single layer step."""
    from paper_2406_17660_amd.block import GrassBlock, RewarmSchedule
    hidden, inter = workloads.BLOCKS[args.block]
    T = args.tokens or cfg.T
    shapes, groups = workloads.llama_block(hidden, inter)
    dY, X, W = workloads.make_block_inputs(cfg, shapes, groups, "cuda", T=T)
    layout = grass.DY_TxM
    if args.layout == "mxt":
        dY = {name: g.t().contiguous() for name, g in dY.items()}
        layout = grass.DY_MxT
    blk = GrassBlock(shapes, groups, cfg.r, T, cfg.dtype, cfg.method, cfg.replacement,
                     alpha=cfg.alpha, adam=AdamHyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps),
                     seed=workloads.BASE_SEED, layout=layout,
                     concurrent_groups=args.concurrent_groups, store_GC=False)
    sched = RewarmSchedule(base_lr=cfg.lr, K=REFRESH_EVERY, rewarm=REFRESH_EVERY)
    blk.refresh_step(dY, X, W)  # set-up: refresh-step workspaces are allocated outside the timed region
    for _ in range(max(args.warmup, 1)):
        blk.step(dY, X, W)
    torch.cuda.synchronize()
    if args.graph:
        blk.capture(dY, X, W)
    blk.t = 0
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(args.steps):
        blk.train_step(dY, X, W, sched)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b)
    flops = sum(2.0 * l.r * T * l.n for l in blk.layers.values())
    print(json.dumps({
        "metric": "GRASS block steps/s (7 linear layers, refresh every 200 steps included)",
        "value": args.steps / (ms * 1e-3), "unit": "block-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == torch.bfloat16 else "f32", "data": "synthetic",
        "config": {"workload": f"LLaMA-{args.block} block: q,k,v,o {hidden}x{hidden}, gate,up "
                               f"{inter}x{hidden}, down {hidden}x{inter}; T={T}, r={cfg.r}, "
                               f"{cfg.method}{'' if cfg.replacement else '-NR'} row selection, "
                               f"dY stored {args.layout}"
                               f"{', groups on concurrent streams' if args.concurrent_groups else ''}"
                               f"{', regular steps replayed from a HIP graph' if args.graph else ''}",
                   "key": f"{args.block}_block" + ("" if args.layout == "txm" else "_mxt"),
                   "argv": " ".join(sys.argv[1:])},
        "compressed_grad_tflops_incl_gather_and_reduce_and_adam": flops * args.steps / (ms * 1e-3) / 1e12,
    }))


def main():
    args = parse()
    if args.summarise:
        import bench_summarise
        return bench_summarise.main(args.summarise)
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build measures the per-layer GRASS step on ONE GPU; "
                 "--gpus N with N > 1 is not supported (no sharding or collectives are built).")
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    grass.lib()
    if args.config is None:  # a block brings its model's token batch, rank and selection rule
        args.config = {"60m": 2, "350m": 3, "1b": 4}.get(args.block, 5)
    cfg = workloads.CONFIGS[args.config]
    if args.clock_trace:
        return clock_trace(workloads.CONFIGS[5])
    if args.adam_cold:
        return bench_adam_cold(args, cfg)
    if args.block:
        return bench_block(args, cfg)
    L = cfg.layers[args.layer]
    T = args.tokens or cfg.T
    m, n, r = L.m, L.n, cfg.r
    dev = "cuda"

    dY = workloads.make_dY(cfg, args.layer, 0, dev, T=T)
    layout = grass.DY_TxM
    if args.layout == "mxt":
        dY = dY.t().contiguous()
        layout = grass.DY_MxT
    X = workloads.make_X(cfg, args.layer, 0, dev, T=T)
    W = workloads.make_W(cfg, args.layer, dev)
    adam = AdamHyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps)
    st = GrassLayer(m, n, r, T, cfg.dtype, cfg.method, cfg.replacement, alpha=cfg.alpha, adam=adam,
                    seed=workloads.BASE_SEED, side=args.side, layout=layout,
                    state_dtype=torch.bfloat16 if args.adam_state == "bf16" else torch.float32,
                    store_GC=False)

    def run(steps, gemm_events=None, end_events=None, tail_events=None):
        for t in range(steps):
            if t % REFRESH_EVERY == 0 and args.refresh == "one-product":
                st.refresh_step(dY, X, W, reset_state=True)  # no compressed-gradient GEMM in it
            else:
                if t % REFRESH_EVERY == 0:
                    st.refresh(dY, X, reset_state=True)
                st.step(dY, X, W, gemm_events[t] if gemm_events else None,
                        tail_events[t] if tail_events else None)
            if end_events:
                end_events[t].record()

    def run_regular(steps, gemm_events):
        for t in range(steps):
            st.step(dY, X, W, gemm_events[t])

    # set-up: the refresh-step workspaces are allocated outside the timed region
    if args.refresh == "one-product":
        st.refresh_step(dY, X, W)
        st.step(dY, X, W)
    else:
        st.row_statistic(dY, X)
    # One plain device-to-device copy of X (T*n*2 bytes read, as many written): the known-size
    # transfer against which the profiler's FETCH_SIZE / WRITE_SIZE counters are calibrated.
    calib = torch.empty_like(X)
    calib.copy_(X)
    del calib
    run(args.warmup)
    torch.cuda.synchronize()
    settle_launches, settle_first_ms, settle_last_ms = settle(run_regular, args.settle_launches)
    # Which roofline binds the layer: 2 r T n flops against the T (m + n) input elements that have
    # to be read once (dY stored T x m: the gather touches every sector of it).  Above the ridge
    # (2500 TFLOP/s / 8 TB/s = 312 flop/B) the dominant kernel, the GEMM, is priced against the
    # matrix cores; below it the whole regular step is priced against HBM.
    esz = 2 if cfg.dtype == torch.bfloat16 else 4
    flops = 2.0 * r * T * st.n  # st.n = width of the compressed gradient (n, or m for side=cols)
    input_bytes = esz * T * (m + n)
    intensity = flops / input_bytes
    mfma_bound = cfg.dtype == torch.bfloat16 and intensity >= PEAK_BF16_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    # Per-kernel events inside the timed region only where the dominant kernel is what is priced:
    # a launch that carries events costs the host tens of microseconds, which a step of a narrow
    # layer (two kernels of 10 - 50 us) does not hide.  Those layers are priced on the whole step;
    # their kernels are timed in a pass of their own after the timed region.
    instrument = mfma_bound
    want_tail = args.side == "rows"  # the fused tail's own start and end (no such hook in column form)
    gemm_events = [(ev(), ev()) for _ in range(args.steps)] if instrument else None
    end_events = [ev() for _ in range(args.steps)]
    tail_events = [(ev(), ev()) for _ in range(args.steps)] if instrument and want_tail else None
    torch.cuda.synchronize()
    t_start, t_stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    t_start.record()
    run(args.steps, gemm_events, end_events, tail_events)
    t_stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    total_ms = t_start.elapsed_time(t_stop)
    ms_per_step = total_ms / args.steps
    # steps whose events were recorded: all of them, or the regular ones
    timed = [t for t in range(args.steps)
             if instrument and not (t % REFRESH_EVERY == 0 and args.refresh == "one-product")]
    kernel_times_from = "the timed region"
    if not timed:
        # No kernel events in the timed region (a layer priced on its whole step, or --steps 1,
        # whose one step is the refresh step and runs no compressed-gradient GEMM): time the GEMM
        # and the tail on regular steps after the timed region.
        timed = list(range(30 if not instrument else 5))
        kernel_times_from = f"{len(timed)} regular steps after the timed region"
        gemm_events = [(ev(), ev()) for _ in timed]
        end_events_r = [ev() for _ in timed]
        tail_events = [(ev(), ev()) for _ in timed] if want_tail else None
        for t in timed:
            st.step(dY, X, W, gemm_events[t], tail_events[t] if tail_events else None)
            end_events_r[t].record()
        torch.cuda.synchronize()
        tail_end = end_events_r
    else:
        tail_end = end_events
    gemm_ms = float(np.mean([gemm_events[t][0].elapsed_time(gemm_events[t][1]) for t in timed]))
    # what follows the GEMM inside the step: the fused split-K reduction + Adam + row update.
    # Its own dispatch times where the library can stamp them; else (and in addition) the
    # interval from the end of the GEMM to the end of the step, which includes the launch gap.
    tail_gap_ms = float(np.mean([gemm_events[t][1].elapsed_time(tail_end[t]) for t in timed]))
    tail_ms = (float(np.mean([tail_events[t][0].elapsed_time(tail_events[t][1]) for t in timed]))
               if tail_events else tail_gap_ms)
    # regular steps alone (the timed region holds one refresh step, at t = 0)
    regular = [end_events[t - 1].elapsed_time(end_events[t]) for t in range(1, args.steps)
               if t % REFRESH_EVERY != 0]
    regular_ms = float(np.mean(regular)) if regular else ms_per_step
    if grass.select_status(st.ws_sel) != grass.OK:
        sys.exit("selection reported non-finite row statistics")

    gemm_tflops = flops / (gemm_ms * 1e-3) / 1e12
    out = {
        "metric": "GRASS layer steps/s (refresh every 200 steps included)",
        "value": args.steps / (total_ms * 1e-3),
        "unit": "layer-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == torch.bfloat16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.cid} ({cfg.name}) layer {L.name}: W {m}x{n}, "
                               f"T={T} tokens, r={r}, {cfg.method}"
                               f"{'' if cfg.replacement else '-NR'} selection of {args.side}, dY stored {args.layout}, {args.adam_state} Adam state, "
                               f"refresh every {REFRESH_EVERY} steps",
                   "m": m, "n": n, "T": T, "r": r, "layer": L.name,
                   "key": (L.name if cfg.cid == 5 else f"c{cfg.cid}_{L.name}")
                          + ("" if args.layout == "txm" else "_mxt") + ("" if args.side == "rows" else "_cols"),
                   "argv": " ".join(sys.argv[1:])},
        "roofline": None,  # filled in below
        "settle_launches": settle_launches,
        "settle_gemm_ms_first_batch": settle_first_ms, "settle_gemm_ms_last_batch": settle_last_ms,
        "host_wall_s": wall,
    }
    traffic, traffic_source = measured_traffic(out["config"]["key"], T)
    gemm_name = ("tn_gemm_bf16_direct_kernel<false, false, true, true>" if args.layout == "mxt"
                 else "tn_gemm_bf16_direct_kernel<false, false, false, false>")
    # bytes the one-call step has to move: the inputs once, M and V read and written, the r rows
    # of W read and written (G_C stays in the partial tiles and is never stored)
    step_bytes = input_bytes + r * st.n * (4 * st.M.element_size() + 2 * esz)
    if mfma_bound:
        out["roofline"] = {"bound": "mfma", "kernel": gemm_name + " (compressed-gradient GEMM)",
                           "achieved": gemm_tflops, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                           "frac": gemm_tflops / PEAK_BF16_MFMA_TFLOPS, "traffic": traffic,
                           "traffic_source": traffic_source,
                           "flops_per_launch": flops, "avg_launch_ms": gemm_ms}
    else:
        gbs = step_bytes / (regular_ms * 1e-3) / 1e9
        out["roofline"] = {"bound": "hbm",
                           "kernel": "the regular step as launched by grass_step_group / grass_step_cols: "
                                     "gather of the selected rows, GEMM, fused split-K reduction + Adam + update",
                           "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": gbs / PEAK_HBM_GBS, "traffic": traffic, "traffic_source": traffic_source,
                           "bytes_per_launch": step_bytes, "avg_launch_ms": regular_ms,
                           "flop_per_input_byte": intensity,
                           "gemm_kernel_tflops": gemm_tflops, "gemm_kernel_ms": gemm_ms,
                           "gemm_kernel_frac_mfma": gemm_tflops / PEAK_BF16_MFMA_TFLOPS}
    out["regular_step_ms"] = regular_ms
    out["refresh_step_ms"] = t_start.elapsed_time(end_events[0])
    out["refresh_step"] = ("full gradient formed once and kept (fp32), row norms from it, selection, the "
                           "selected rows of it as G_C, Adam + update" if args.refresh == "one-product" else
                           "row norms in the epilogue of the full-gradient GEMM (G not stored), selection, "
                           "then a regular step")
    # The step's tail as it runs inside the step sequence (state and weights come from HBM: a
    # whole GEMM pass lies between two uses): from the event after the GEMM to the end of the step.
    plan_tile, plan_slices = grass.cgrad_plan(T, st.n, r, st.dt, layout, m=st.m)
    tail_bytes = r * st.n * (4 * plan_slices + 4 * st.M.element_size() + 2 * esz)
    out["step_tail"] = {"what": "split-K reduction + Adam + update after the GEMM, inside the step "
                                "(fused kernel; for column selection plus the column update)",
                        "ms": tail_ms, "timed_over": kernel_times_from,
                        "timed_by": ("the kernel dispatch's own start and end" if tail_events
                                                    else "events after the GEMM and at the end of the step"),
                        "ms_from_end_of_gemm_to_end_of_step": tail_gap_ms,
                        "k_slices": plan_slices, "algorithmic_bytes": tail_bytes,
                        "GBs": tail_bytes / (tail_ms * 1e-3) / 1e9,
                        "frac_hbm": tail_bytes / (tail_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}

    if not args.no_extras and cfg.dtype == torch.bfloat16:
        # Context for the fraction above: what kernels of nothing but this matrix instruction
        # sustain on this very machine.  The clock under that load depends on the box and on what
        # the instructions are fed: constants; values distributed like the GEMM's inputs (dY-like
        # on the left, X-like on the right) held in registers; the same values read from LDS
        # fragment by fragment as the GEMM reads its operands (no global memory traffic).
        g = torch.Generator(device=dev)
        g.manual_seed(workloads.BASE_SEED + 99)
        vals = torch.randn(32768, generator=g, device=dev)
        left = (torch.arange(32768, device=dev) // 2048) % 8 < 4
        vals = torch.where(left, vals * 0.1, vals).to(torch.bfloat16)
        from paper_2406_17660_amd import probe as mfma_probe  # measurement aid, a library of its own
        probe = mfma_probe.mfma_rate(source=mfma_probe.CONSTANTS)
        probe_regs = mfma_probe.mfma_rate(source=mfma_probe.REGISTERS, operands=vals)
        probe_lds = mfma_probe.mfma_rate(source=mfma_probe.LDS, operands=vals)
        out["matrix_core_context"] = {
            "mfma_only_kernel_tflops_this_box": probe,
            "mfma_only_kernel_normal_operands_tflops": probe_regs,
            "mfma_plus_lds_reads_kernel_normal_operands_tflops": probe_lds,
            "gemm_frac_of_mfma_only_kernel": gemm_tflops / probe,
            "gemm_frac_of_mfma_only_kernel_normal_operands": gemm_tflops / probe_regs,
            "gemm_frac_of_mfma_plus_lds_reads_kernel": gemm_tflops / probe_lds}

    if not args.no_extras and args.side == "rows" and args.layout == "txm":
        detail = {}
        it = 20
        med, mn = time_calls(lambda: st.compressed_grad(dY, X), it, warmup=5)
        detail["compressed_grad_call_ms"] = med  # pack + GEMM + split-K reduce
        detail["compressed_grad_call_min_ms"] = mn
        detail["compressed_grad_call_tflops"] = flops / (med * 1e-3) / 1e12
        # What the memory system of this machine delivers for plain streams (datasheet: 8 TB/s):
        # a device copy (1 read + 1 write) and a triad-like add (2 reads + 1 write) of 1 GiB arrays.
        a1 = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev)
        a2 = torch.empty_like(a1)
        med, _ = time_calls(lambda: a2.copy_(a1), 10)
        copy_gbs = 2 * a1.numel() * 4 / (med * 1e-3) / 1e9
        med, _ = time_calls(lambda: torch.add(a1, a2, out=a2), 10)
        triad_gbs = 3 * a1.numel() * 4 / (med * 1e-3) / 1e9
        del a1, a2
        detail["hbm_measured_copy_GBs"] = copy_gbs
        detail["hbm_measured_triad_GBs"] = triad_gbs

        # Adam + scatter, warm (the same 100 MB every call: it stays in the 256 MB last-level
        # cache) and cold (eight sets of state and weights, 0.8 GB, cycled between calls)
        st.adam_t = 0
        med, mn = time_calls(lambda: st.adam_scatter(W), 100, warmup=10)
        esz = 2 if cfg.dtype == torch.bfloat16 else 4
        ab = r * n * (4 + 4 * st.M.element_size() + 2 * esz)
        detail["adam_scatter_ms"] = med
        detail["adam_scatter_min_ms"] = mn
        detail["adam_scatter_GBs"] = ab / (med * 1e-3) / 1e9
        detail["adam_scatter_frac_hbm"] = detail["adam_scatter_GBs"] / PEAK_HBM_GBS
        detail["adam_scatter_frac_measured_triad"] = detail["adam_scatter_GBs"] / triad_gbs
        a = st.adam
        sets = [(torch.randn_like(st.GC), torch.zeros_like(st.M), torch.zeros_like(st.V),
                 W.clone()) for _ in range(8)]
        turn = [0]

        def cold_adam():
            g_, m_, v_, w_ = sets[turn[0] % len(sets)]
            turn[0] += 1
            grass.adam_scatter(g_, m_, v_, a.lr, a.beta1, a.beta2, a.eps, 1 + turn[0], w_, st.idx,
                               st.rho, st.alpha)
        med, mn = time_calls(cold_adam, 40, warmup=8)
        detail["adam_scatter_cold_ms"] = med
        detail["adam_scatter_cold_GBs"] = ab / (med * 1e-3) / 1e9
        detail["adam_scatter_cold_frac_hbm"] = detail["adam_scatter_cold_GBs"] / PEAK_HBM_GBS
        del sets

        med, _ = time_calls(lambda: st.row_statistic(dY, X), 5, warmup=1)
        detail["refresh_statistic_fused_ms"] = med  # full-gradient GEMM with the squares in its epilogue
        st.full_gradient(dY, X)
        med, mn = time_calls(lambda: grass.row_stats(st.G, st.sumsq), it)
        gb = m * n * st.G.element_size() + 4 * m
        detail["row_stats_ms"] = med
        detail["row_stats_min_ms"] = mn
        detail["row_stats_GBs"] = gb / (med * 1e-3) / 1e9
        detail["row_stats_frac_hbm"] = detail["row_stats_GBs"] / PEAK_HBM_GBS
        copies = [st.G.clone() for _ in range(max(2, int(600e6 // max(gb, 1))))]  # > 256 MB in total

        def cold_stats():
            turn[0] += 1
            grass.row_stats(copies[turn[0] % len(copies)], st.sumsq)
        med, _ = time_calls(cold_stats, 40, warmup=len(copies))
        detail["row_stats_cold_ms"] = med
        detail["row_stats_cold_GBs"] = gb / (med * 1e-3) / 1e9
        detail["row_stats_cold_frac_hbm"] = detail["row_stats_cold_GBs"] / PEAK_HBM_GBS
        del copies
        grass.row_stats(st.G, st.sumsq)
        med, _ = time_calls(lambda: grass.select_rows(st.sumsq, r, st.method, st.replacement,
                                                      st.scale, st.seed, 0, st.idx, st.rho,
                                                      st.ws_sel), it)
        detail["select_rows_ms"] = med
        med_dense, _ = time_calls(lambda: st.full_gradient(dY, X), 5, warmup=1)
        tmp = torch.empty((r, n), dtype=torch.float32, device=dev)
        med_g, _ = time_calls(lambda: grass.gather_rows(st.G, st.idx, st.rho, tmp), it)
        detail["naive_full_grad_ms"] = med_dense
        detail["naive_full_grad_tflops"] = 2.0 * m * T * n / (med_dense * 1e-3) / 1e12
        detail["naive_gather_ms"] = med_g
        detail["speedup_vs_naive_full_G_then_gather"] = (med_dense + med_g) / detail[
            "compressed_grad_call_ms"]
        detail["regular_step_ms"] = detail["compressed_grad_call_ms"] + detail["adam_scatter_ms"]
        # a refresh step with two products = statistic + selection + zeroing the state + the
        # regular step (sum of the parts); with one product: measured as a whole
        med, _ = time_calls(lambda: (st.M.zero_(), st.V.zero_()), it)
        detail["refresh_step_two_products_ms"] = (detail["refresh_statistic_fused_ms"]
                                                  + detail["select_rows_ms"] + med
                                                  + detail["regular_step_ms"])
        med, _ = time_calls(lambda: st.refresh_step(dY, X, W), 5, warmup=1)
        detail["refresh_step_one_product_ms"] = med
        detail["amortised_step_ms_K200"] = (199 * detail["regular_step_ms"]
                                            + detail["refresh_step_one_product_ms"]) / 200
        # What a plain stream of the Adam kernel's size reaches when its data is cold: a + b -> c
        # over r x n fp32 arrays (12 B per element), eight sets cycled.  Kernels of tens of
        # microseconds do not reach the rates of the 1 GiB streams above.
        trio = [tuple(torch.empty((r, n), dtype=torch.float32, device=dev).normal_() for _ in range(3))
                for _ in range(8)]

        def cold_add():
            turn[0] += 1
            x_, y_, z_ = trio[turn[0] % len(trio)]
            torch.add(x_, y_, out=z_)
        med, _ = time_calls(cold_add, 40, warmup=8)
        detail["hbm_measured_cold_add_same_size_GBs"] = 12.0 * r * n / (med * 1e-3) / 1e9
        del trio
        if args.config == 5 and args.layer == 0 and T == cfg.T:
            # the other three layers of the configuration, in the same launch configuration
            detail["other_layers"] = [layer_figures(cfg, k) for k in range(1, len(cfg.layers))]
        detail["paper_context"] = ("paper: 13B LLaMA half-precision pretraining on one 40 GB "
                                   "A100; no per-layer timing is published")
        out["detail"] = detail

    if (not args.no_cpu_baseline and args.side == "rows" and args.adam_state == "f32"
            and args.layout == "txm"):
        out["cpu_baseline"] = cpu_baseline(cfg, L, dY, X, st, W, args.cpu_seconds)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
