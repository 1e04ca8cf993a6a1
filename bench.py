#!/usr/bin/env python3
"""Benchmark of the DS-Sync hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, all
resident in HBM before the clock starts:
    ds_partition (host)  ->  ds_group_sync (GPU)  ->  ds_consensus (GPU)
The headline workload is configuration 3 of the benchmark set: W = 32 workers
in groups of 8, P = 25,557,032 fp32 parameters per replica (ResNet-50-sized),
gradients g_i = c_i (mu + 0.5 z_i), seed 2, lr 0.01, a new division every step.

Prints ONE JSON line.  ``value`` is the algorithmic bytes of a step
(16 B per worker-element: read x, read g, write x, read x again for the
consensus pass) divided by the wall-clock step time.  ``roofline`` is for the
dominant kernel, the fused group-sync (12 B per worker-element), timed with
events on the stream it is launched on.  ``all_configs`` holds a shorter run of
each of the five benchmark configurations (kernel times as mean, median and
minimum over the timed steps).  ``cpu_baseline`` is the CPU oracle on the host
cores, a reported figure only.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
PROBE_SRC = os.path.join(ROOT, "bench_probe.hip")
PROBE_LIB = os.path.join(ROOT, "libbench_probe.so")
KERNEL_SRC = os.path.join(ROOT, "paper_2007_03298_amd", "csrc", "group_sync.hip")


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


def device_clocks():
    """Clocks and memory bus of the current device as the HIP runtime reports them (through the probe library;
    empty if that is not built): context for the assumed peak, which stays the published 8 TB/s."""
    import ctypes
    if not os.path.exists(PROBE_LIB):
        return {}
    lib = ctypes.CDLL(PROBE_LIB)
    mem, sclk, bus = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    if not hasattr(lib, "bench_probe_device_clocks") or \
            lib.bench_probe_device_clocks(ctypes.byref(mem), ctypes.byref(sclk), ctypes.byref(bus)) != 0:
        return {}
    return {"memory_clock_MHz": mem.value / 1e3 or None, "shader_clock_MHz": sclk.value / 1e3 or None,
            "memory_bus_bits": bus.value or None}


def git_blob_id(path: str) -> str:
    """What `git hash-object` prints for the file: identifies the kernel source a record belongs to."""
    with open(path, "rb") as fh:
        data = fh.read()
    return hashlib.sha1(b"blob %d\0" % len(data) + data).hexdigest()


def measured_traffic(name: str, workload: str):
    """HBM bytes per launch of the dominant kernel, from the rocprofv3 counter
    runs recorded under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by
    what the same counter reads for the plain copy kernel).  The counters
    cannot be read from inside this process, so the figure is the recorded one;
    it is reported only for the workload and layout it was measured on and only
    while the kernel source is the one it was measured with (null otherwise)."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as fh:
            rec = json.load(fh)
        if rec.get("workload") != workload or rec.get("kernel_source_blob") != git_blob_id(KERNEL_SRC):
            return None
        return rec.get("hbm_bytes_per_launch")
    except (OSError, ValueError):
        return None


def host_info():
    model, mem_kib = "unknown", 0
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
        with open("/proc/meminfo") as fh:
            for line in fh:
                if line.startswith("MemTotal"):
                    mem_kib = int(line.split()[1])
                    break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {"nproc": usable, "cpu_model": model, "ram_GiB": round(mem_kib / 2**20, 1)}


def cpu_baseline(cfg, Xh, Gh, budget_s: float = 10.0, max_iters: int = 200):
    """The oracle, as it stands, on the host cores: whole configuration-3 stacks,
    as many iterations as fit in about ``budget_s`` seconds of wall clock with all
    of its threads, then a short leg on one thread."""
    import oracle
    W, P = Xh.shape

    def leg(limit_s, min_iters, t_base):
        t_step = t_cons = 0.0
        iters = 0
        while iters < max_iters and (iters < min_iters or t_step + t_cons < limit_s):
            a = time.perf_counter()
            perm, off = oracle.partition(cfg.seed, t_base + iters, W, cfg.sizes)
            oracle.step(Xh, Gh, perm, off, cfg.lr)
            b = time.perf_counter()
            oracle.consensus(Xh)
            c = time.perf_counter()
            t_step += b - a
            t_cons += c - b
            iters += 1
        return iters, t_step, t_cons

    threads = oracle.num_threads()
    iters, t_step, t_cons = leg(budget_s, 4, 1000)
    total = t_step + t_cons
    oracle.set_num_threads(1)
    try:
        iters1, t_step1, t_cons1 = leg(4.0, 1, 2000)
    finally:
        oracle.set_num_threads(threads)
    total1 = t_step1 + t_cons1
    out = {
        "value": round(16.0 * W * P * iters / total / 1e9, 3),
        "unit": "GB/s",
        "cores": threads,
        "kind": "oracle",
        "sample": "all %d columns x %d workers of the same workload, %d iterations "
                  "(partition + step + consensus), %.1f s wall" % (P, W, iters, total),
        "ms_per_step": round(total / iters * 1e3, 2),
        "group_sync_ms": round(t_step / iters * 1e3, 2),
        "consensus_ms": round(t_cons / iters * 1e3, 2),
        "single_thread": {"value": round(16.0 * W * P * iters1 / total1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                          "sample": "the same stacks, %d iteration(s), %.1f s wall" % (iters1, total1),
                          "ms_per_step": round(total1 / iters1 * 1e3, 1),
                          "group_sync_ms": round(t_step1 / iters1 * 1e3, 1),
                          "consensus_ms": round(t_cons1 / iters1 * 1e3, 1)},
    }
    out.update(host_info())
    return out


def spread(ms):
    """Mean, median and minimum of a list of per-step milliseconds."""
    return {"ms": round(statistics.fmean(ms), 4), "ms_median": round(statistics.median(ms), 4),
            "ms_min": round(min(ms), 4)}


class Workload:
    """Stacks, division stream and launch closures of one benchmark configuration."""

    def __init__(self, idx, dev, args):
        import torch
        import paper_2007_03298_amd as ds
        from paper_2007_03298_amd import workloads as wl
        self.torch, self.ds, self.idx, self.wl = torch, ds, idx, wl
        cfg = self.cfg = wl.CONFIGS[idx]
        self.W = W = cfg.W
        if cfg.ragged:
            # layer list of configuration 5: only the columns inside the segments are work
            self.segs, self.ld, _ = wl.ragged_segments(cfg.seed)
            self.P = sum(n for _, n in self.segs)
            self.plan_bytes = ds.ds_ragged_plan_bytes(self.segs)
            self.plan = torch.empty(self.plan_bytes, dtype=torch.uint8, device=dev)
            self.packed = ds.pack_segments(self.segs)
            self.plan_id = ds.ds_ragged_plan(self.packed, self.ld, self.ld, self.plan, self.plan_bytes)
        else:
            self.segs = None
            self.P = cfg.P
            self.ld = self.P if args.dense_rows else wl.padded_ld(self.P)   # rows on 1-KiB boundaries
        self.g_bytes = 2 if cfg.bf16_grads else 4
        self.g_dtype = ds.DS_BF16 if cfg.bf16_grads else ds.DS_F32
        run = wl.Run(cfg, dev, P=self.ld, ld=self.ld)
        # the replica stack is allocated BETWEEN the two resident gradient stacks, so that either of them is one
        # stack away from it: at 35 GB per stack a stack two away lies in another third of the HBM more often
        g_torch = torch.bfloat16 if cfg.bf16_grads else torch.float32
        g_first = torch.empty(W, self.ld, dtype=g_torch, device=dev)
        x_mid = torch.empty(W, self.ld, dtype=torch.float32, device=dev)
        g_last = torch.empty(W, self.ld, dtype=g_torch, device=dev)
        self.X = run.init_params(out=x_mid)                 # same draws in the same order as without `out`
        self.use_v = args.local_opt in ("momentum", "both")
        self.use_s = args.local_opt in ("swa", "both")
        self.Gs = [run.gradients(out=g_first), run.gradients(out=g_last)]   # resident in HBM, used in turn
        self.tiled = bool(getattr(args, "tiled", False)) and not cfg.ragged
        self.ts = W * wl.TILE                               # tile stride of the tiled variant
        if self.tiled:
            self.X = wl.to_tiled(self.X, self.P)
            for j in range(len(self.Gs)):
                self.Gs[j] = wl.to_tiled(self.Gs[j], self.P)
            torch.cuda.empty_cache()
        self.V = torch.zeros_like(self.X) if self.use_v else None
        self.S = self.X.clone() if self.use_s else None
        self.weight_decay = 5e-4 if self.use_v else 0.0
        pitch = self.ts if self.tiled else self.ld
        self.opt = (ds.local_opt(self.V, pitch, 0.9, self.weight_decay, self.S, pitch, 0.9)
                    if (self.use_v or self.use_s) else None)
        self.P_cons = self.ld if cfg.ragged else self.P    # ragged: the norm runs over the whole arena
        self.ws_bytes = ds.ds_consensus_workspace_bytes(W, self.P_cons)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
        self.dev_out = torch.zeros(W, dtype=torch.float64, device=dev)
        self.stream = torch.cuda.current_stream()
        self.layerwise = None
        self.sync_bytes = (8.0 + self.g_bytes + 8.0 * self.use_v + 8.0 * self.use_s) * W * self.P
        self.cons_bytes = 4.0 * W * self.P_cons

    def use_layerwise(self, n_streams):
        self.layerwise = self.ds.LayerwiseSync(self.segs, n_streams) if n_streams > 0 else None

    def step(self, t, ev=None):
        ds, cfg, st = self.ds, self.cfg, self.stream
        perm, off = ds.ds_partition(cfg.seed, t, self.W, cfg.sizes)
        G = self.Gs[t % len(self.Gs)]
        if ev:
            ev[0].record(st)
        if self.layerwise is not None:
            # Sec. V-A1: one launch per layer, last layer first, on side streams; here all layers are
            # ready at once and the main stream waits for all of them
            self.layerwise.backward(self.X, G, self.g_dtype, self.ld, self.ld, self.W, perm, off, cfg.lr,
                                    V=self.V, ldv=self.ld, momentum=0.9 if self.use_v else 0.0,
                                    weight_decay=self.weight_decay, S=self.S, lds=self.ld, swa_factor=0.9, stream=st)
            self.layerwise.wait_all(st)
        elif cfg.ragged:
            ds.ds_group_sync_ragged_opt(self.X, G, self.g_dtype, self.packed, self.ld, self.ld, self.W, perm, off,
                                        cfg.lr, self.opt, self.plan, self.plan_bytes, self.plan_id, st)
        elif self.tiled:
            ds.ds_group_sync_tiled(self.X, G, self.g_dtype, self.P, self.ts, self.ts, self.W, perm, off, cfg.lr,
                                   self.opt, st)
        else:
            ds.ds_group_sync_opt(self.X, G, self.g_dtype, self.P, self.ld, self.ld, self.W, perm, off, cfg.lr,
                                 self.opt, st)
        if ev:
            ev[1].record(st)
        if self.tiled:
            ds.ds_consensus_tiled(self.X, self.P, self.ts, self.W, self.dev_out, self.ws, self.ws_bytes, st)
        else:
            ds.ds_consensus(self.X, self.P_cons, self.ld, self.W, self.dev_out, self.ws, self.ws_bytes, st)
        if ev:
            ev[2].record(st)

    def timed(self, warmup, steps, t0=0):
        """`warmup` untimed steps, then `steps` timed ones: wall clock per step and per-kernel event times."""
        torch = self.torch
        self.first_timed_t = t0 + warmup
        for t in range(warmup):
            self.step(t0 + t)
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        torch.cuda.synchronize()
        a = time.perf_counter()
        for k in range(steps):
            self.step(t0 + warmup + k, events[k])
        torch.cuda.synchronize()
        b = time.perf_counter()
        sync_ms = [e[0].elapsed_time(e[1]) for e in events]
        cons_ms = [e[1].elapsed_time(e[2]) for e in events]
        return (b - a) / steps * 1e3, sync_ms, cons_ms

    def fused_timed(self, warmup, steps, t0=5000):
        """The step and the norms of its result in one pass (ds_group_sync_consensus): reported
        separately, never in `value`, whose consensus term stays the full second pass."""
        torch, ds, cfg = self.torch, self.ds, self.cfg
        if cfg.ragged or self.opt is not None or self.tiled:
            return None
        n_groups = len(cfg.sizes)
        need = ds.ds_group_sync_consensus_workspace_bytes(self.P, n_groups)
        ws = torch.empty(need, dtype=torch.uint8, device=self.X.device)
        out = torch.zeros(self.W, dtype=torch.float64, device=self.X.device)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        for k in range(warmup + steps):
            t = t0 + k
            perm, off = ds.ds_partition(cfg.seed, t, self.W, cfg.sizes)
            if k == warmup:
                torch.cuda.synchronize()
                a = time.perf_counter()
                ev[0].record(self.stream)
            ds.ds_group_sync_consensus(self.X, self.Gs[t % len(self.Gs)], self.g_dtype, self.P, self.ld, self.ld,
                                       self.W, perm, off, cfg.lr, out, ws, need, self.stream)
            if k >= warmup:
                ev[k - warmup + 1].record(self.stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - a) / steps * 1e3
        ms = [ev[k].elapsed_time(ev[k + 1]) for k in range(steps)]
        # the full pass on the same state, for the gap between the two ways to the norms
        ds.ds_consensus(self.X, self.P_cons, self.ld, self.W, self.dev_out, self.ws, self.ws_bytes, self.stream)
        torch.cuda.synchronize()
        gap = float((out - self.dev_out).abs().max() / self.dev_out.abs().max().clamp_min(1e-300))
        rec = spread(ms)
        rec.update(ms_per_step=round(wall, 4), bytes_moved=int(self.sync_bytes),
                   GBps=round(self.sync_bytes / (rec["ms_median"] * 1e-3) / 1e9, 1),
                   max_rel_gap_to_full_consensus=gap,
                   note="ds_group_sync_consensus: step and norms in one pass over the stacks (the norms come from "
                        "the group means, the stack is not read again); not in value")
        return rec

    def tiled_timed(self, warmup, steps, t0=7000):
        """The same step and consensus pass on TILED stacks (the W pieces of a 256-column tile
        contiguous; ds_group_sync_tiled, ds_consensus_tiled, ds_group_sync_consensus_tiled).
        Another layout of the same workload: reported separately, never in `value`.
        Converts this workload's stacks, so it runs last."""
        torch, ds, cfg, wl = self.torch, self.ds, self.cfg, self.wl
        if cfg.ragged or self.opt is not None or self.tiled:
            return None
        W, P, st = self.W, self.P, self.stream
        ts = self.ts
        self.X = wl.to_tiled(self.X, P)
        for j in range(len(self.Gs)):
            self.Gs[j] = wl.to_tiled(self.Gs[j], P)
            torch.cuda.empty_cache()
        n_groups = len(cfg.sizes)
        need = ds.ds_group_sync_consensus_workspace_bytes(P, n_groups)
        ws2 = torch.empty(need, dtype=torch.uint8, device=self.X.device)
        out2 = torch.zeros(W, dtype=torch.float64, device=self.X.device)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        fe = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        for k in range(warmup + steps):
            perm, off = ds.ds_partition(cfg.seed, t0 + k, W, cfg.sizes)
            if k == warmup:
                torch.cuda.synchronize()
                a = time.perf_counter()
            e = ev[k - warmup] if k >= warmup else None
            if e:
                e[0].record(st)
            ds.ds_group_sync_tiled(self.X, self.Gs[k % len(self.Gs)], self.g_dtype, P, ts, ts, W, perm, off, cfg.lr,
                                   None, st)
            if e:
                e[1].record(st)
            ds.ds_consensus_tiled(self.X, P, ts, W, self.dev_out, self.ws, self.ws_bytes, st)
            if e:
                e[2].record(st)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - a) / steps * 1e3
        for k in range(5 + steps):
            perm, off = ds.ds_partition(cfg.seed, t0 + 500 + k, W, cfg.sizes)
            if k == 5:
                fe[0].record(st)
            ds.ds_group_sync_consensus_tiled(self.X, self.Gs[k % len(self.Gs)], self.g_dtype, P, ts, ts, W, perm, off,
                                             cfg.lr, out2, ws2, need, st)
            if k >= 5:
                fe[k - 4].record(st)
        ds.ds_consensus_tiled(self.X, P, ts, W, self.dev_out, self.ws, self.ws_bytes, st)
        torch.cuda.synchronize()
        gap = float((out2 - self.dev_out).abs().max() / self.dev_out.abs().max().clamp_min(1e-300))
        # one row per group, valid because the last call above was a step with this division
        ge = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
        for k in range(11):
            ds.ds_consensus_grouped_tiled(self.X, P, ts, W, perm, off, out2, self.ws, self.ws_bytes, st)
            ge[k].record(st)
        torch.cuda.synchronize()
        grouped_ms = statistics.median(ge[k].elapsed_time(ge[k + 1]) for k in range(10))
        grouped_gap = float((out2 - self.dev_out).abs().max() / self.dev_out.abs().max().clamp_min(1e-300))
        sync = spread([e[0].elapsed_time(e[1]) for e in ev])
        cons = spread([e[1].elapsed_time(e[2]) for e in ev])
        fused = spread([fe[k].elapsed_time(fe[k + 1]) for k in range(steps)])
        sync["GBps"] = round(self.sync_bytes / (sync["ms"] * 1e-3) / 1e9, 1)
        cons["GBps"] = round(4.0 * W * P / (cons["ms"] * 1e-3) / 1e9, 1)
        fused["GBps"] = round(self.sync_bytes / (fused["ms_median"] * 1e-3) / 1e9, 1)
        fused["max_rel_gap_to_full_consensus"] = gap
        return {"tile_stride": ts, "ms_per_step": round(wall, 4),
                "GBps": round((self.sync_bytes + 4.0 * W * P) / (wall * 1e-3) / 1e9, 1),
                "group_sync": sync, "consensus": cons, "fused_step_and_consensus": fused,
                "consensus_grouped": {"ms": round(grouped_ms, 4), "max_rel_gap_to_full": grouped_gap},
                "note": "the same workload with the stacks stored tile by tile (element (i, p) at "
                        "(p // 256) * W * 256 + i * 256 + p % 256): another layout, not in value"}

    def record(self, ms_step, sync_ms, cons_ms):
        """Figures of one configuration for `all_configs`."""
        sync, cons = spread(sync_ms), spread(cons_ms)
        sync_gbps = self.sync_bytes / (sync["ms"] * 1e-3) / 1e9
        cons_gbps = self.cons_bytes / (cons["ms"] * 1e-3) / 1e9
        sync.update(GBps=round(sync_gbps, 1), frac=round(sync_gbps / HBM_PEAK_GBPS, 4),
                    bytes_per_launch=int(self.sync_bytes))
        cons.update(GBps=round(cons_gbps, 1), frac=round(cons_gbps / HBM_PEAK_GBPS, 4),
                    bytes_per_launch=int(self.cons_bytes))
        # the two resident gradient stacks are used in turn: where the stacks lie in HBM shows at 35 GB per stack
        n = len(self.Gs)
        sync["ms_by_gradient_stack"] = [round(statistics.fmean(sync_ms[(j - self.first_timed_t) % n::n]), 4)
                                        for j in range(n)]
        rec = {"workload": self.cfg.name, "W": self.W, "group_size": self.cfg.group, "P": self.P, "ld": self.ld,
               "ms_per_step": round(ms_step, 4),
               "GBps": round((self.sync_bytes + self.cons_bytes) / (ms_step * 1e-3) / 1e9, 1),
               "group_sync": sync, "consensus": cons}
        if self.idx == 1:
            rec["note"] = ("cache-resident (33.6 MB stacks) and launch-bound: not an HBM figure; GB/s can exceed "
                           "what HBM delivers")
        return rec

    def free(self):
        for name in ("X", "V", "S", "Gs", "ws", "plan", "opt"):
            setattr(self, name, None)
        self.torch.cuda.empty_cache()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30,
                    help="untimed steps first; the first ~25 steps after start-up run about 8 %% slower")
    ap.add_argument("--config", type=int, default=0,
                    help="time only this benchmark configuration (1-5) as the headline; default: configuration 3, "
                         "the one the metric is quoted on, followed by a shorter run of all five (`all_configs`)")
    ap.add_argument("--no-all-configs", action="store_true", help="skip the shorter runs of all five configurations")
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
                    help="leading dimension = P (rows start inside a cache line) instead of P rounded up to an "
                         "odd multiple of 256 elements (rows on 1-KiB boundaries)")
    ap.add_argument("--tiled", action="store_true",
                    help="configurations 1-4: the stacks stored tile by tile (the W pieces of a 256-column tile "
                         "contiguous) and the *_tiled entry points instead of the row-major layout; a variant, "
                         "so no recorded traffic is attached")
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

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    headline = args.config if args.config else 3
    variant = args.local_opt != "none" or args.layerwise > 0 or args.dense_rows or args.graph > 0 or args.tiled
    want_all = not args.config and not args.no_all_configs and not variant
    wk = Workload(headline, dev, args)
    cfg, W, P, ld = wk.cfg, wk.W, wk.P, wk.ld
    if args.layerwise > 0:
        if not cfg.ragged:
            print("bench.py: --layerwise needs --config 5", file=sys.stderr)
            return 2
        wk.use_layerwise(args.layerwise)
    stream = wk.stream

    probe = None
    if args.probe_copy > 0:
        probe_copy = load_probe()
        Y = torch.empty_like(wk.X)
        nbytes = wk.X.numel() * 4
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(args.probe_copy + 1)]
        probe_copy(Y, wk.X, nbytes, stream)
        pe[0].record(stream)
        for k in range(args.probe_copy):
            probe_copy(Y, wk.X, nbytes, stream)
            pe[k + 1].record(stream)
        torch.cuda.synchronize()
        pms = sum(pe[k].elapsed_time(pe[k + 1]) for k in range(args.probe_copy)) / args.probe_copy
        probe = {"bytes_read": nbytes, "bytes_written": nbytes, "ms": round(pms, 4),
                 "GBps": round(2.0 * nbytes / (pms * 1e-3) / 1e9, 1)}
        del Y

    ms_step, sync_list, cons_list = wk.timed(args.warmup, args.steps)
    sync_ms, cons_ms = statistics.fmean(sync_list), statistics.fmean(cons_list)

    # reported separately, never part of `value`: the norm from one row per group, valid because the
    # step has just made the members of every group identical
    grouped = None
    if not wk.tiled:
        perm, off = ds.ds_partition(cfg.seed, args.warmup + args.steps - 1, W, cfg.sizes)
        ge = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
        dev_grouped = torch.zeros(W, dtype=torch.float64, device=dev)
        ds.ds_consensus_grouped(wk.X, wk.P_cons, ld, W, perm, off, dev_grouped, wk.ws, wk.ws_bytes, stream)
        ge[0].record(stream)
        for k in range(10):
            ds.ds_consensus_grouped(wk.X, wk.P_cons, ld, W, perm, off, dev_grouped, wk.ws, wk.ws_bytes, stream)
            ge[k + 1].record(stream)
        torch.cuda.synchronize()
        grouped_ms = sum(ge[k].elapsed_time(ge[k + 1]) for k in range(10)) / 10
        grouped_gap = float((dev_grouped - wk.dev_out).abs().max() / wk.dev_out.abs().max().clamp_min(1e-300))
        grouped = {"ms": round(grouped_ms, 4), "bytes_read": int(4.0 * len(cfg.sizes) * wk.P_cons),
                   "note": "one row per group; valid right after a group-sync; not in value",
                   "max_rel_gap_to_full": grouped_gap}

    graph_replay = None
    if args.graph > 0 and wk.layerwise is None:
        graphs = []
        for k in range(args.graph):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                wk.stream = torch.cuda.current_stream()       # the capturing stream
                wk.step(k)
            graphs.append(g)
        wk.stream = stream
        for k in range(args.warmup):
            graphs[k % args.graph].replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for k in range(args.steps):
            graphs[k % args.graph].replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - g0) / args.steps * 1e3
        graph_replay = {"graphs": args.graph, "ms_per_step": round(g_ms, 4)}

    sync_bytes, cons_bytes = wk.sync_bytes, wk.cons_bytes
    sync_gbps = sync_bytes / (sync_ms * 1e-3) / 1e9
    cons_gbps = cons_bytes / (cons_ms * 1e-3) / 1e9
    value = (sync_bytes + cons_bytes) / (ms_step * 1e-3) / 1e9
    d = wk.dev_out.cpu()
    props = torch.cuda.get_device_properties(0)

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
        "group_sync": dict(spread(sync_list), GBps=round(sync_gbps, 1),
                           pct_of_hbm_peak=round(100.0 * sync_gbps / HBM_PEAK_GBPS, 2),
                           # drift over the timed region, and the two resident gradient stacks apart
                           ms_by_quarter=[round(statistics.fmean(sync_list[q * len(sync_list) // 4:
                                                                           max((q + 1) * len(sync_list) // 4,
                                                                               q * len(sync_list) // 4 + 1)]), 4)
                                          for q in range(4)],
                           ms_by_gradient_stack=[round(statistics.fmean(sync_list[(j - wk.first_timed_t) % 2::2]), 4) for j in range(2)]
                           if len(sync_list) >= 2 else None),
        "consensus": dict(spread(cons_list), GBps=round(cons_gbps, 1),
                          pct_of_hbm_peak=round(100.0 * cons_gbps / HBM_PEAK_GBPS, 2),
                          max_deviation=float(d.max())),
        "roofline": {"bound": "hbm", "kernel": "group_sync_kernel<float, flat>", "bytes_per_launch": int(sync_bytes),
                     "achieved": round(sync_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(sync_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic("group_sync_cfg%d_traffic.txt" % headline,
                                                 "cfg%d W=%d g=%d P=%d ld=%d" % (headline, W, cfg.group, P, ld))},
        "device": {"name": props.name or getattr(props, "gcnArchName", ""), "arch": getattr(props, "gcnArchName", ""),
                   "compute_units": props.multi_processor_count, "hbm_GiB": round(props.total_memory / 2**30, 1),
                   "assumed_hbm_peak_GBps": HBM_PEAK_GBPS, **device_clocks()},
    }
    if grouped is not None:
        out["consensus_grouped"] = grouped
    if wk.tiled:
        out["config"]["layout"] = "tiled"
        out["config"]["tile_stride"] = wk.ts
        out["roofline"]["kernel"] = "group_sync_kernel<float, tiled>"
        out["roofline"]["traffic"] = None
    if probe is not None:
        out["probe_copy"] = probe
    if graph_replay is not None:
        graph_replay["GBps"] = round((sync_bytes + cons_bytes) / (graph_replay["ms_per_step"] * 1e-3) / 1e9, 1)
        graph_replay["note"] = "the same step replayed from HIP graphs, one per division of a periodic list; not in value"
        out["graph_replay"] = graph_replay
    if wk.opt is not None:
        out["config"]["local_opt"] = args.local_opt
        out["roofline"]["kernel"] += " + " + args.local_opt
        out["roofline"]["traffic"] = None
    if wk.layerwise is not None:
        out["config"]["layerwise_streams"] = args.layerwise
        out["config"]["launches_per_step"] = len(wk.segs)
        out["roofline"]["traffic"] = None
    if cfg.ragged:
        out["dtype"] = "f32 (bf16 gradients)"
        out["roofline"]["kernel"] = "group_sync_kernel<bf16, ragged>"

    cpu_inputs = None
    if not args.no_cpu_baseline and not cfg.ragged and wk.opt is None and headline != 4 and not wk.tiled:
        import numpy as np
        cpu_inputs = (cfg, np.ascontiguousarray(wk.X[:, :P].cpu().numpy()),
                      np.ascontiguousarray(wk.Gs[0][:, :P].cpu().numpy()))

    if want_all:
        # a shorter run of every configuration (the headline one included, under the same short protocol)
        steps_all, warm_all = max(10, min(args.steps, 30)), max(5, min(args.warmup, 15))
        allc = {}
        wk.free()
        for idx in (1, 2, 3, 4, 5):
            free, _ = torch.cuda.mem_get_info()
            w2 = None
            try:
                w2 = Workload(idx, dev, args)
                rec = w2.record(*w2.timed(warm_all, steps_all))
                rec["steps"], rec["warmup"] = steps_all, warm_all
                fused = w2.fused_timed(5, steps_all)
                if fused is not None:
                    rec["fused_step_and_consensus"] = fused
                if idx == 5:
                    # Sec. V-A1 / IV-A: the same step as one launch per layer on K side streams
                    lw = {}
                    for K in (1, 2):
                        w2.use_layerwise(K)
                        ms_k, sync_k, _ = w2.timed(3, 10, t0=1000)
                        lw["streams_%d" % K] = dict(spread(sync_k), ms_per_step=round(ms_k, 4))
                    w2.use_layerwise(0)
                    lw["launches_per_step"] = len(w2.segs)
                    lw["single_launch_ms"] = rec["group_sync"]["ms"]
                    lw["note"] = "one launch per layer in reverse order with one event per layer; not in value"
                    rec["layerwise"] = lw
                tiled = w2.tiled_timed(5, steps_all)
                if tiled is not None:
                    rec["tiled_layout"] = tiled
                allc[str(idx)] = rec
            except torch.OutOfMemoryError:
                allc[str(idx)] = {"skipped": "not enough free HBM (%.0f GB free)" % (free / 1e9)}
            finally:
                if w2 is not None:
                    w2.free()
                del w2
        out["all_configs"] = allc

    if cpu_inputs is not None:
        out["cpu_baseline"] = cpu_baseline(*cpu_inputs)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
