"""The step under HIP graph capture.

The paper's group list is periodic (Listing 1: ``groupList[t % len(groupList)]``;
Sec. IV-B2: ``W_k = W_{k+B}``), and no entry point of the library allocates,
frees, synchronises or clears memory with a memset, so one iteration
(group-sync + consensus) can be captured once per entry of the list and the
training loop then replays B graphs in turn: the launch-bound case of small
models pays one graph launch per step instead of three kernel launches.

Each replay is checked bit for bit against the same calls made eagerly on a
copy of the state, with eager work and synchronisations between the replays,
and the final state against the CPU oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_03298_amd as ds
from test_gpu_parity import DEV, TOL_F32, scaled_error

pytestmark = pytest.mark.gpu


def test_periodic_group_list_replayed_from_hip_graphs():
    rack_of = [0, 0, 0, 0, 1, 1, 1, 1]                 # the paper's two-rack testbed (Sec. V-A5)
    none8, none2 = [0] * 8, [0, 0]
    W, P, lr = 8, 70001, 0.01
    ld = ds.ds_padded_ld(P)
    B = ds.ds_pattern_period(rack_of, none2, none8)
    assert B >= 2
    gen = torch.Generator(device=DEV).manual_seed(11)
    X = torch.empty(W, ld, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=gen)
    G = torch.empty(W, ld, dtype=torch.float32, device=DEV)          # static gradient buffer of the graphs
    need = ds.ds_consensus_workspace_bytes(W, P)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    dev = torch.zeros(W, dtype=torch.float64, device=DEV)

    # eager twin: same calls on copies
    Xe, wse, deve = X.clone(), torch.empty_like(ws), torch.zeros_like(dev)
    # oracle's own trajectory
    Xo = X.cpu().numpy().copy()

    def step(Xs, ws_, out, perm, off):
        ds.ds_group_sync(Xs, G, ds.DS_F32, P, ld, ld, W, perm, off, lr)
        ds.ds_consensus(Xs, P, ld, W, out, ws_, need)

    parts = [ds.ds_pattern(rack_of, none2, none8, k) for k in range(B)]
    # first launches load the kernels; keep that out of the capture
    G.normal_(generator=gen)
    scratch = X.clone()
    for perm, off in parts:
        step(scratch, ws, dev, perm, off)
    torch.cuda.synchronize()

    graphs = []
    for perm, off in parts:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(X, ws, dev, perm, off)
        graphs.append(g)
    torch.cuda.synchronize()

    for t in range(3 * B + 1):
        G.normal_(generator=gen)                       # eager work between the replays
        Gh = G.cpu().numpy()                           # (synchronises)
        perm, off = parts[t % B]
        graphs[t % B].replay()
        step(Xe, wse, deve, perm, off)
        torch.cuda.synchronize()
        assert torch.equal(X.view(torch.int32), Xe.view(torch.int32)), "replay %d differs from the eager step" % t
        assert torch.equal(dev.view(torch.int64), deve.view(torch.int64))
        oracle.step(Xo, Gh, perm, off, lr, 0, P)
    assert scaled_error(X.cpu().numpy()[:, :P], Xo[:, :P]) <= TOL_F32
    np.testing.assert_allclose(dev.cpu().numpy(), oracle.consensus(Xo, P), rtol=1e-5)


def _states(W, P, ld, seed, tiled):
    """Two identical sets of buffers (one for the graph, one for the eager twin)."""
    from paper_2007_03298_amd import workloads as wl
    gen = torch.Generator(device=DEV).manual_seed(seed)
    X = torch.empty(W, ld, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=gen)
    V = torch.empty(W, ld, dtype=torch.float32, device=DEV).normal_(generator=gen)
    S = torch.empty(W, ld, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=gen)
    if tiled:
        X, V, S = (wl.to_tiled(t, P) for t in (X, V, S))
    out = []
    for _ in range(2):
        out.append({"X": X.clone(), "V": V.clone(), "S": S.clone(),
                    "norms": torch.zeros(W, dtype=torch.float64, device=DEV),
                    "ws": torch.empty(ds.ds_consensus_workspace_bytes(W, P), dtype=torch.uint8, device=DEV),
                    "ws2": torch.empty(ds.ds_group_sync_consensus_workspace_bytes(P, 8), dtype=torch.uint8, device=DEV)})
    return out


@pytest.mark.parametrize("which", ["extended", "ragged", "one_pass", "static", "tiled", "tiled_one_pass"])
def test_every_launch_only_entry_point_replays_from_a_hip_graph(which):
    # none of them allocates, copies, synchronises or clears memory, so each can be captured; every replay
    # must equal the same call made eagerly on a twin of the state, with eager work and waits in between
    from paper_2007_03298_amd import workloads as wl
    W, P, lr = 16, 9001, 0.01
    ld = ds.ds_padded_ld(P)
    tiled = which.startswith("tiled")
    ts = W * 256
    graph_state, eager_state = _states(W, P, ld, 21, tiled)
    gen = torch.Generator(device=DEV).manual_seed(22)
    G_rows = torch.empty(W, ld, dtype=torch.float32, device=DEV).normal_(generator=gen)
    G = wl.to_tiled(G_rows, P) if tiled else G_rows                  # static gradient buffer of the graph
    perm, off = ds.ds_partition(9, 0, W, [3, 5, 8])
    segs = [(0, 300), (512, 2049), (4096, 4000)]
    plan_bytes = ds.ds_ragged_plan_bytes(segs)
    plan = torch.empty(plan_bytes, dtype=torch.uint8, device=DEV)
    plan_id = ds.ds_ragged_plan(segs, ld, ld, plan, plan_bytes)

    def call(st):
        pitch = ts if tiled else ld
        opt = ds.local_opt(st["V"], pitch, 0.9, 1e-3, st["S"], pitch, 0.8)
        need, need2 = st["ws"].numel(), st["ws2"].numel()
        if which == "extended":
            ds.ds_group_sync_opt(st["X"], G, ds.DS_F32, P, ld, ld, W, perm, off, lr, opt)
            ds.ds_consensus_grouped(st["X"], P, ld, W, perm, off, st["norms"], st["ws"], need)
        elif which == "ragged":
            ds.ds_group_sync_ragged_opt(st["X"], G, ds.DS_F32, segs, ld, ld, W, perm, off, lr, opt, plan, plan_bytes, plan_id)
        elif which == "one_pass":
            ds.ds_group_sync_consensus(st["X"], G, ds.DS_F32, P, ld, ld, W, perm, off, lr, st["norms"], st["ws2"], need2)
        elif which == "static":
            ds.ds_group_sync(st["X"], G, ds.DS_F32, P, ld, ld, W, perm, off, lr)
            ds.ds_consensus_static(st["X"], P, ld, W, st["norms"])
        elif which == "tiled":
            ds.ds_group_sync_tiled(st["X"], G, ds.DS_F32, P, ts, ts, W, perm, off, lr, opt)
            ds.ds_consensus_tiled(st["X"], P, ts, W, st["norms"], st["ws"], need)
        else:
            ds.ds_group_sync_consensus_tiled(st["X"], G, ds.DS_F32, P, ts, ts, W, perm, off, lr, st["norms"], st["ws2"], need2)

    # first launches load the kernels; keep that out of the capture (on a state of its own)
    call(_states(W, P, ld, 23, tiled)[0])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(graph_state)
    torch.cuda.synchronize()
    for t in range(4):
        fresh = torch.empty(W, ld, dtype=torch.float32, device=DEV).normal_(generator=gen)   # eager work between replays
        G.copy_(wl.to_tiled(fresh, P) if tiled else fresh)
        torch.cuda.synchronize()
        g.replay()
        call(eager_state)
        torch.cuda.synchronize()
        for name in ("X", "V", "S"):
            assert torch.equal(graph_state[name].view(torch.int32), eager_state[name].view(torch.int32)), (which, t, name)
        assert torch.equal(graph_state["norms"].view(torch.int64), eager_state["norms"].view(torch.int64)), (which, t)


def test_no_entry_point_changes_the_free_device_memory():
    # "allocates nothing": after the kernels are loaded, a round of calls to every GPU entry point leaves the
    # device's free memory exactly where it was (hipMemGetInfo, which sees every allocation of the process)
    from paper_2007_03298_amd import workloads as wl
    W, P, lr = 16, 9001, 0.01
    ld = ds.ds_padded_ld(P)
    ts = W * 256
    st, _ = _states(W, P, ld, 31, False)
    tt, _ = _states(W, P, ld, 32, True)
    G = torch.empty(W, ld, dtype=torch.float32, device=DEV).normal_()
    Gt = wl.to_tiled(G, P)
    Gb = G.to(torch.bfloat16)
    perm, off = ds.ds_partition(9, 0, W, [3, 5, 8])
    segs = [(0, 300), (512, 2049), (4096, 4000)]
    plan_bytes = ds.ds_ragged_plan_bytes(segs)
    plan = torch.empty(plan_bytes, dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream()
    need, need2 = st["ws"].numel(), st["ws2"].numel()

    def round_of_calls():
        plan_id = ds.ds_ragged_plan(segs, ld, ld, plan, plan_bytes)
        opt = ds.local_opt(st["V"], ld, 0.9, 1e-3, st["S"], ld, 0.8)
        opt_t = ds.local_opt(tt["V"], ts, 0.9, 1e-3, tt["S"], ts, 0.8)
        ds.ds_group_sync(st["X"], G, ds.DS_F32, P, ld, ld, W, perm, off, lr)
        ds.ds_group_sync(st["X"], Gb, ds.DS_BF16, P, ld, ld, W, perm, off, lr, stream=side)
        side.synchronize()
        ds.ds_group_sync_opt(st["X"], G, ds.DS_F32, P, ld, ld, W, perm, off, lr, opt)
        ds.ds_group_sync_ragged(st["X"], G, ds.DS_F32, segs, ld, ld, W, perm, off, lr, plan, plan_bytes, plan_id)
        ds.ds_group_sync_ragged_opt(st["X"], Gb, ds.DS_BF16, segs, ld, ld, W, perm, off, lr, opt, plan, plan_bytes, plan_id)
        ds.ds_consensus(st["X"], P, ld, W, st["norms"], st["ws"], need)
        ds.ds_consensus_static(st["X"], P, ld, W, st["norms"])
        ds.ds_consensus_grouped(st["X"], P, ld, W, perm, off, st["norms"], st["ws"], need)
        ds.ds_group_sync_consensus(st["X"], G, ds.DS_F32, P, ld, ld, W, perm, off, lr, st["norms"], st["ws2"], need2)
        ds.ds_group_sync_tiled(tt["X"], Gt, ds.DS_F32, P, ts, ts, W, perm, off, lr, opt_t)
        ds.ds_consensus_tiled(tt["X"], P, ts, W, tt["norms"], tt["ws"], need)
        ds.ds_consensus_grouped_tiled(tt["X"], P, ts, W, perm, off, tt["norms"], tt["ws"], need)
        ds.ds_group_sync_consensus_tiled(tt["X"], Gt, ds.DS_F32, P, ts, ts, W, perm, off, lr, tt["norms"], tt["ws2"], need2)
        torch.cuda.synchronize()

    round_of_calls()                                   # loads the kernels, resolves the static array's address
    free_before, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        round_of_calls()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before
