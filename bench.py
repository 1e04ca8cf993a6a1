#!/usr/bin/env python3
"""Benchmark of the DS-Sync hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, all
resident in HBM before the clock starts:
    ds_partition (host)  ->  ds_group_sync (GPU)  ->  ds_consensus (GPU)
The workload is configuration 3 of the benchmark set: W = 32 workers in groups
of 8, P = 25,557,032 fp32 parameters per replica (ResNet-50-sized), gradients
g_i = c_i (mu + 0.5 z_i), seed 2, lr 0.01, a new division every step.

Prints ONE JSON line.  ``value`` is the algorithmic bytes of a step
(16 B per worker-element: read x, read g, write x, read x again for the
consensus pass) divided by the wall-clock step time.  ``roofline`` is for the
dominant kernel, the fused group-sync (12 B per worker-element), timed with
events on the stream it is launched on.  ``cpu_baseline`` is the CPU oracle on
the host cores, a reported figure only.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
PROBE_SRC = os.path.join(ROOT, "bench_probe.hip")
PROBE_LIB = os.path.join(ROOT, "libbench_probe.so")


def build_probe() -> str:
    """Compile the plain copy kernel that serves as yardstick (bench_probe.hip, gfx950)."""
    from paper_2007_03298_amd.build import compile_shared
    return compile_shared([PROBE_SRC], PROBE_LIB)


def load_probe():
    """The copy kernel as ``probe_copy(dst, src, nbytes, stream)``; it must have been built."""
    import ctypes
    if not os.path.exists(PROBE_LIB):
        raise RuntimeError("libbench_probe.so is not built: run `python bench.py --build-probe`")
    lib = ctypes.CDLL(PROBE_LIB)
    lib.bench_probe_copy.restype = ctypes.c_int
    lib.bench_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]

    def probe_copy(dst, src, nbytes, stream):
        rc = lib.bench_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream)
        if rc != 0:
            raise RuntimeError("bench_probe_copy failed: %d" % rc)
    return probe_copy


def measured_traffic(name: str, workload: str):
    """HBM bytes per launch of the dominant kernel, from the rocprofv3 counter
    runs recorded under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by
    what the same counter reads for the plain copy kernel).  The counters
    cannot be read from inside this process, so the figure is the recorded one
    and is reported only for the workload and layout it was measured on."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as fh:
            rec = json.load(fh)
        return rec.get("hbm_bytes_per_launch") if rec.get("workload") == workload else None
    except (OSError, ValueError):
        return None


def cpu_baseline(cfg, X, G, budget_s: float = 10.0, max_iters: int = 200):
    """The oracle, as it stands, on the host cores: whole configuration-3 stacks,
    as many iterations as fit in about ``budget_s`` seconds of wall clock."""
    import numpy as np
    import oracle
    W, P = cfg.W, cfg.P
    Xh = np.ascontiguousarray(X[:, :P].cpu().numpy())
    Gh = np.ascontiguousarray(G[:, :P].cpu().numpy())
    t_step = t_cons = 0.0
    iters = 0
    while iters < max_iters and (iters < 4 or t_step + t_cons < budget_s):
        a = time.perf_counter()
        perm, off = oracle.partition(cfg.seed, 1000 + iters, W, cfg.sizes)
        oracle.step(Xh, Gh, perm, off, cfg.lr)
        b = time.perf_counter()
        oracle.consensus(Xh)
        c = time.perf_counter()
        t_step += b - a
        t_cons += c - b
        iters += 1
    total = t_step + t_cons
    return {
        "value": round(16.0 * W * P * iters / total / 1e9, 3),
        "unit": "GB/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "all %d columns x %d workers of the same workload, %d iterations "
                  "(partition + step + consensus), %.1f s wall" % (P, W, iters, total),
        "ms_per_step": round(total / iters * 1e3, 2),
        "group_sync_ms": round(t_step / iters * 1e3, 2),
        "consensus_ms": round(t_cons / iters * 1e3, 2),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30,
                    help="untimed steps first; the first ~25 steps after start-up run about 8 %% slower")
    ap.add_argument("--config", type=int, default=3,
                    help="benchmark configuration 1-5 (default 3, the one the headline metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--local-opt", choices=["none", "momentum", "swa", "both"], default="none",
                    help="time the extended step (momentum 0.9 / weight decay 5e-4 buffers and/or the SWA "
                         "moving average, +8 B per worker-column each) instead of the plain one")
    ap.add_argument("--layerwise", type=int, default=0, metavar="K",
                    help="configuration 5 only: synchronise layer by layer, one launch per segment in reverse "
                         "layer order, round-robin over K streams with one event per layer (the shape of the "
                         "paper's backward-hook / pre-forward-hook overlap) instead of the single ragged launch")
    ap.add_argument("--graph", type=int, default=0, metavar="K",
                    help="also capture K steps (the divisions of iterations 0..K-1, a periodic group list as in "
                         "the paper's Listing 1) as HIP graphs and time their replay; reported as `graph_replay`, "
                         "never as `value` (pays off where the step is launch-bound, i.e. configuration 1)")
    ap.add_argument("--dense-rows", action="store_true",
                    help="leading dimension = P (rows not 256-byte aligned) instead of P rounded up to 64")
    ap.add_argument("--probe-copy", type=int, default=0, metavar="N",
                    help="also launch the plain copy kernel N times on a stack-sized buffer before the "
                         "timed region (yardstick for bandwidth and for profiler counter scaling)")
    ap.add_argument("--build-probe", action="store_true", help="compile bench_probe.hip and exit")
    args = ap.parse_args()
    if args.build_probe:
        print(build_probe())
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (W simulated workers stacked in one HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch
    import paper_2007_03298_amd as ds
    from paper_2007_03298_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    cfg = wl.CONFIGS[args.config]
    W = cfg.W
    if cfg.ragged:
        # layer list of configuration 5: only the columns inside the segments are work
        segs, ld, _ = wl.ragged_segments(cfg.seed)
        P = sum(n for _, n in segs)
        plan_bytes = ds.ds_ragged_plan_bytes(segs)
        plan = torch.empty(plan_bytes, dtype=torch.uint8, device=dev)
        packed = ds.pack_segments(segs)
        plan_id = ds.ds_ragged_plan(packed, ld, ld, plan, plan_bytes)
    else:
        P = cfg.P
        ld = P if args.dense_rows else wl.padded_ld(P)   # rows start on 256-byte boundaries
    g_bytes = 2 if cfg.bf16_grads else 4
    run = wl.Run(cfg, dev, P=ld, ld=ld)
    X = run.init_params()
    use_v = args.local_opt in ("momentum", "both")
    use_s = args.local_opt in ("swa", "both")
    V = torch.zeros_like(X) if use_v else None
    S = X.clone() if use_s else None
    opt = ds.local_opt(V, ld, 0.9, 5e-4 if use_v else 0.0, S, ld, 0.9) if (use_v or use_s) else None
    n_grad = 2                                   # gradient stacks resident in HBM, used in turn
    Gs = [run.gradients() for _ in range(n_grad)]
    P_cons = ld if cfg.ragged else P              # ragged: the norm runs over the whole arena
    ws_bytes = ds.ds_consensus_workspace_bytes(W, P_cons)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    dev_out = torch.zeros(W, dtype=torch.float64, device=dev)
    stream = torch.cuda.current_stream()

    side = [torch.cuda.Stream() for _ in range(args.layerwise)] if args.layerwise > 0 else []
    if side and not cfg.ragged:
        print("bench.py: --layerwise needs --config 5", file=sys.stderr)
        return 2
    layer_done = [torch.cuda.Event() for _ in segs] if side else []

    def layerwise(t, perm, off):
        # Sec. V-A1: the backward hook of a layer updates it locally and starts its synchronisation
        # without blocking; the pre-forward hook waits for that layer's event.  Layers become ready
        # from the last to the first; here all are ready at once and the main stream waits for all.
        fork = torch.cuda.Event()
        fork.record(stream)
        for st in side:
            st.wait_event(fork)
        G = Gs[t % n_grad]
        for k, s in enumerate(reversed(range(len(segs)))):
            o, n = segs[s]
            st = side[k % len(side)]
            ds.ds_group_sync_opt(X.data_ptr() + 4 * o, G.data_ptr() + g_bytes * o, ds.DS_BF16, n, ld, ld, W,
                                 perm, off, cfg.lr, None, st)
            layer_done[s].record(st)
        for e in layer_done:
            stream.wait_event(e)

    def step(t, ev=None):
        perm, off = ds.ds_partition(cfg.seed, t, W, cfg.sizes)
        if ev:
            ev[0].record(stream)
        if side:
            layerwise(t, perm, off)
        elif cfg.ragged:
            ds.ds_group_sync_ragged_opt(X, Gs[t % n_grad], ds.DS_BF16, packed, ld, ld, W, perm, off, cfg.lr, opt,
                                        plan, plan_bytes, plan_id, stream)
        else:
            ds.ds_group_sync_opt(X, Gs[t % n_grad], ds.DS_F32, P, ld, ld, W, perm, off, cfg.lr, opt, stream)
        if ev:
            ev[1].record(stream)
        ds.ds_consensus(X, P_cons, ld, W, dev_out, ws, ws_bytes, stream)
        if ev:
            ev[2].record(stream)

    probe = None
    if args.probe_copy > 0:
        probe_copy = load_probe()
        Y = torch.empty_like(X)
        nbytes = X.numel() * 4
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(args.probe_copy + 1)]
        probe_copy(Y, X, nbytes, stream)
        pe[0].record(stream)
        for k in range(args.probe_copy):
            probe_copy(Y, X, nbytes, stream)
            pe[k + 1].record(stream)
        torch.cuda.synchronize()
        pms = sum(pe[k].elapsed_time(pe[k + 1]) for k in range(args.probe_copy)) / args.probe_copy
        probe = {"bytes_read": nbytes, "bytes_written": nbytes, "ms": round(pms, 4),
                 "GBps": round(2.0 * nbytes / (pms * 1e-3) / 1e9, 1)}
        del Y

    for t in range(args.warmup):
        step(t)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(args.warmup + k, events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    # reported separately, never part of `value`: the norm from one row per group, valid because the
    # step has just made the members of every group identical
    perm, off = ds.ds_partition(cfg.seed, args.warmup + args.steps - 1, W, cfg.sizes)
    ge = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
    dev_grouped = torch.zeros(W, dtype=torch.float64, device=dev)
    ds.ds_consensus_grouped(X, P_cons, ld, W, perm, off, dev_grouped, ws, ws_bytes, stream)
    ge[0].record(stream)
    for k in range(10):
        ds.ds_consensus_grouped(X, P_cons, ld, W, perm, off, dev_grouped, ws, ws_bytes, stream)
        ge[k + 1].record(stream)
    torch.cuda.synchronize()
    grouped_ms = sum(ge[k].elapsed_time(ge[k + 1]) for k in range(10)) / 10
    grouped_gap = float((dev_grouped - dev_out).abs().max() / dev_out.abs().max().clamp_min(1e-300))

    graph_replay = None
    if args.graph > 0 and not side:
        graphs = []
        for k in range(args.graph):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                stream = torch.cuda.current_stream()       # the capturing stream
                step(k)
            graphs.append(g)
        stream = torch.cuda.current_stream()
        for k in range(args.warmup):
            graphs[k % args.graph].replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for k in range(args.steps):
            graphs[k % args.graph].replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - g0) / args.steps * 1e3
        graph_replay = {"graphs": args.graph, "ms_per_step": round(g_ms, 4)}

    ms_step = (t1 - t0) / args.steps * 1e3
    sync_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps
    cons_ms = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps
    sync_bytes = (8.0 + g_bytes + 8.0 * use_v + 8.0 * use_s) * W * P
    cons_bytes = 4.0 * W * P_cons
    sync_gbps = sync_bytes / (sync_ms * 1e-3) / 1e9
    cons_gbps = cons_bytes / (cons_ms * 1e-3) / 1e9
    value = (sync_bytes + cons_bytes) / (ms_step * 1e-3) / 1e9
    d = dev_out.cpu()

    out = {
        "metric": "DS-Sync step (partition + fused group-sync + consensus) algorithmic HBM GB/s",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": cfg.name, "W": W, "group_size": cfg.group, "P": P, "ld": ld, "lr": cfg.lr,
                   "seed": cfg.seed, "bytes_per_step": int(sync_bytes + cons_bytes)},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "group_sync": {"ms": round(sync_ms, 4), "GBps": round(sync_gbps, 1),
                       "pct_of_hbm_peak": round(100.0 * sync_gbps / HBM_PEAK_GBPS, 2)},
        "consensus": {"ms": round(cons_ms, 4), "GBps": round(cons_gbps, 1),
                      "pct_of_hbm_peak": round(100.0 * cons_gbps / HBM_PEAK_GBPS, 2),
                      "max_deviation": float(d.max())},
        "consensus_grouped": {"ms": round(grouped_ms, 4), "bytes_read": int(4.0 * len(cfg.sizes) * P_cons),
                              "note": "one row per group; valid right after a group-sync; not in value",
                              "max_rel_gap_to_full": grouped_gap},
        "roofline": {"bound": "hbm", "kernel": "group_sync_kernel<float, flat>", "bytes_per_launch": int(sync_bytes),
                     "achieved": round(sync_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(sync_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic("group_sync_cfg%d_traffic.txt" % args.config,
                                                 "cfg%d W=%d g=%d P=%d ld=%d" % (args.config, W, cfg.group, P, ld))},
    }
    if probe is not None:
        out["probe_copy"] = probe
    if graph_replay is not None:
        graph_replay["GBps"] = round((sync_bytes + cons_bytes) / (graph_replay["ms_per_step"] * 1e-3) / 1e9, 1)
        graph_replay["note"] = "the same step replayed from HIP graphs, one per division of a periodic list; not in value"
        out["graph_replay"] = graph_replay
    if opt is not None:
        out["config"]["local_opt"] = args.local_opt
        out["roofline"]["kernel"] += " + " + args.local_opt
        out["roofline"]["traffic"] = None
    if side:
        out["config"]["layerwise_streams"] = len(side)
        out["config"]["launches_per_step"] = len(segs)
    if cfg.ragged:
        out["dtype"] = "f32 (bf16 gradients)"
        out["roofline"]["kernel"] = "group_sync_kernel<bf16, ragged>"
    if not args.no_cpu_baseline and not cfg.ragged and opt is None:
        out["cpu_baseline"] = cpu_baseline(cfg, X, Gs[0])
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
