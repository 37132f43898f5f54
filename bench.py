#!/usr/bin/env python3
"""Benchmark of the GRASS layer step on one MI355X.

One "step" is one pass of Algorithm 1 for one linear layer over one synthetic token batch
that is already resident in HBM: on steps with t = 0 (mod K, K = 200 as in the paper's
pretraining runs) the refresh work (row statistic of the full gradient, taken in the epilogue
of the full-gradient GEMM so that G itself is not stored; selection; state reset), and on
every step the compressed gradient, Adam on r x n, and the scatter into W.  The
timed region starts at t = 0, so it always contains exactly one refresh per 200 steps.

Prints ONE JSON line: metric, value (layer steps per second), ms_per_step, the workload, a
`roofline` object for the dominant kernel (the compressed-gradient GEMM, timed with HIP events
around its launches) and a `cpu_baseline` object (the fp64 oracle on the host cores, on a bounded
sample).  Only one GPU is supported.
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


def measured_traffic(layer_name, T):
    """HBM bytes per launch of the GEMM kernel as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE (profiles/gemm_traffic.json, written from those runs); None if not recorded
    for this workload."""
    path = os.path.join(ROOT, "profiles", "gemm_traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path)).get(f"{layer_name}:T={T}")
    return rec["bytes_per_launch"] if rec else None


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
    blk.refresh(dY, X)  # set-up: refresh-step workspaces are allocated outside the timed region
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
                               f"{', regular steps replayed from a HIP graph' if args.graph else ''}"},
        "compressed_grad_tflops_incl_gather_and_reduce_and_adam": flops * args.steps / (ms * 1e-3) / 1e12,
    }))


def main():
    args = parse()
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

    def run(steps, gemm_events=None):
        for t in range(steps):
            if t % REFRESH_EVERY == 0:
                st.refresh(dY, X, reset_state=True)
            st.step(dY, X, W, gemm_events[t] if gemm_events else None)

    st.row_statistic(dY, X)  # set-up: allocates the refresh-step workspace outside the timed region
    # One plain device-to-device copy of X (T*n*2 bytes read, as many written): the known-size
    # transfer against which the profiler's FETCH_SIZE / WRITE_SIZE counters are calibrated.
    calib = torch.empty_like(X)
    calib.copy_(X)
    del calib
    run(args.warmup)
    torch.cuda.synchronize()
    gemm_events = [(ev(), ev()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start, t_stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    t_start.record()
    run(args.steps, gemm_events)
    t_stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    total_ms = t_start.elapsed_time(t_stop)
    ms_per_step = total_ms / args.steps
    gemm_ms = float(np.mean([a.elapsed_time(b) for a, b in gemm_events]))
    if grass.select_status(st.ws_sel) != grass.OK:
        sys.exit("selection reported non-finite row statistics")

    flops = 2.0 * r * T * st.n  # st.n = width of the compressed gradient (n, or m for side=cols)
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
                   "m": m, "n": n, "T": T, "r": r},
        "roofline": {"bound": "mfma",
                     "kernel": ("tn_gemm_bf16_direct_kernel<false, false, true, true>" if args.layout == "mxt"
                                else "tn_gemm_bf16_direct_kernel<false, false, false, false>") + " (compressed-gradient GEMM)",
                     "achieved": gemm_tflops, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / PEAK_BF16_MFMA_TFLOPS,
                     "traffic": measured_traffic(L.name, T) if args.layout == "txm" else None,
                     "flops_per_launch": flops, "avg_launch_ms": gemm_ms},
        "host_wall_s": wall,
    }

    if not args.no_extras:
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
        out["roofline"]["mfma_only_kernel_tflops_this_box"] = probe
        out["roofline"]["mfma_only_kernel_normal_operands_tflops"] = probe_regs
        out["roofline"]["mfma_plus_lds_reads_kernel_normal_operands_tflops"] = probe_lds
        out["roofline"]["frac_of_mfma_only_kernel"] = gemm_tflops / probe
        out["roofline"]["frac_of_mfma_only_kernel_normal_operands"] = gemm_tflops / probe_regs
        out["roofline"]["frac_of_mfma_plus_lds_reads_kernel"] = gemm_tflops / probe_lds

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
        # a refresh step = statistic + selection + zeroing the state + the regular step
        med, _ = time_calls(lambda: (st.M.zero_(), st.V.zero_()), it)
        detail["refresh_step_ms"] = (detail["refresh_statistic_fused_ms"] + detail["select_rows_ms"]
                                     + med + detail["regular_step_ms"])
        detail["amortised_step_ms_K200"] = (199 * detail["regular_step_ms"]
                                            + detail["refresh_step_ms"]) / 200
        detail["paper_context"] = ("paper: 13B LLaMA half-precision pretraining on one 40 GB "
                                   "A100; no per-layer timing is published")
        out["detail"] = detail

    if (not args.no_cpu_baseline and args.side == "rows" and args.adam_state == "f32"
            and args.layout == "txm"):
        out["cpu_baseline"] = cpu_baseline(cfg, L, dY, X, st, W, args.cpu_seconds)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
