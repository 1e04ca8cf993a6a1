"""Randomised GPU parity over every way into the step: row-major, tiled and
ragged stacks, the one-pass step+norms on both layouts, any division of 1..64
workers, both gradient types, optional momentum and SWA state, tile strides
and pitches with slack - each case against the CPU oracle, followed by the
consensus entry points of its layout on the state the GPU holds."""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_03298_amd as ds
from paper_2007_03298_amd import workloads as wl
from test_gpu_parity import DEV, TOL_F32, scaled_error

pytestmark = pytest.mark.gpu

LAYOUTS = ["flat", "tiled", "ragged", "fused", "fused_tiled"]


def random_segments(r):
    """Disjoint segments on multiples of 8 columns, in shuffled order; returns (segments, ld)."""
    segs, at = [], 8 * int(r.integers(0, 5))
    for _ in range(int(r.integers(1, 12))):
        n = int(r.choice([0, 1, 7, 8, 255, 256, 300, 2047, 2048, 2049, 5000])) if r.integers(0, 2) else int(r.integers(0, 6000))
        segs.append((at, n))
        at = (at + n + 7) // 8 * 8 + 8 * int(r.integers(0, 4))
    r.shuffle(segs)
    return [(int(o), int(n)) for o, n in segs], max((at + 3) // 4 * 4, 8)


@pytest.mark.parametrize("seed", range(150))
def test_random_case_any_layout(seed):
    r = np.random.default_rng(880000 + seed)
    W = int(r.integers(1, 65))
    cuts = sorted(set(r.integers(1, W, size=int(r.integers(0, min(W, 9)))).tolist())) if W > 1 else []
    edges = [0] + cuts + [W]
    sizes = [b - a for a, b in zip(edges[:-1], edges[1:])]
    layout = LAYOUTS[seed % len(LAYOUTS)]
    tiled, fused = layout in ("tiled", "fused_tiled"), layout in ("fused", "fused_tiled")
    bf16 = bool(r.integers(0, 2))
    use_v = bool(r.integers(0, 2)) and not fused
    use_s = bool(r.integers(0, 2)) and not fused
    # columns: tile edges and arbitrary counts (rows of 1 or 2 columns are hand-picked cases elsewhere)
    P = int(r.choice([3, 4, 5, 255, 256, 257, 1023, 1025, 2047, 2048, 2049, 4099, 9001, 20000, 70001])) if r.integers(0, 3) \
        else int(r.integers(3, 40000))
    lr, mu, f = float(r.choice([0.0, 0.01, 0.1])), 0.9, 0.8
    wd = 0.0 if fused else float(r.choice([0.0, 1e-3]))       # the one-pass step+norms is the plain step
    dt = ds.DS_BF16 if bf16 else ds.DS_F32
    case = "W=%d sizes=%s %s bf16=%s V=%s S=%s P=%d" % (W, sizes, layout, bf16, use_v, use_s, P)
    g = torch.Generator(device=DEV).manual_seed(seed)
    pad = lambda n: (n + 3) // 4 * 4 + 4 * int(r.integers(0, 20))
    if layout == "ragged":
        segs, ld = random_segments(r)
        ldx = ldg = ldv = lds = ld
    else:
        ldx, ldg, ldv, lds = pad(P), pad(P), pad(P), pad(P)
    X = torch.empty(W, ldx, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=g)
    G = torch.empty(W, ldg, dtype=torch.float32, device=DEV).normal_(generator=g)
    if bf16:
        G = G.to(torch.bfloat16)
    V = torch.empty(W, ldv, dtype=torch.float32, device=DEV).normal_(generator=g) if use_v else None
    S = torch.empty(W, lds, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=g) if use_s else None
    Gh = wl.tensor_to_numpy(G)
    if tiled:
        tsx, tsg, tsv, tss = (W * 256 + 256 * int(r.integers(0, 3)) for _ in range(4))
        Xt, Gt = wl.to_tiled(X, P, tsx), wl.to_tiled(G, P, tsg)
        Vt = wl.to_tiled(V, P, tsv) if use_v else None
        St = wl.to_tiled(S, P, tss) if use_s else None
        opt = ds.local_opt(Vt, tsv, mu, wd, St, tss, f)
        host = lambda T, ts: wl.tensor_to_numpy(wl.from_tiled(T, P, W, ts))
    else:
        opt = ds.local_opt(V, ldv, mu, wd, S, lds, f)
    if layout == "ragged":
        plan_bytes = ds.ds_ragged_plan_bytes(segs)
        plan = torch.empty(max(plan_bytes, 16), dtype=torch.uint8, device=DEV)
        plan_id = ds.ds_ragged_plan(segs, ldx, ldg, plan, plan_bytes) if plan_bytes else 0
    for t in range(2):
        perm, off = ds.ds_partition(seed, t, W, sizes)
        if tiled:
            Xo = host(Xt, tsx)[:, :P].copy()
            Vo = host(Vt, tsv)[:, :P].copy() if use_v else None
            So = host(St, tss)[:, :P].copy() if use_s else None
            Go = np.ascontiguousarray(Gh[:, :P])
        else:
            Xo, Go = wl.tensor_to_numpy(X), Gh
            Vo = wl.tensor_to_numpy(V) if use_v else None
            So = wl.tensor_to_numpy(S) if use_s else None
        before = Xo.copy()
        norms = None
        if layout == "flat":
            ds.ds_group_sync_opt(X, G, dt, P, ldx, ldg, W, perm, off, lr, opt)
        elif layout == "tiled":
            ds.ds_group_sync_tiled(Xt, Gt, dt, P, tsx, tsg, W, perm, off, lr, opt)
        elif layout == "ragged":
            if plan_bytes:
                ds.ds_group_sync_ragged_opt(X, G, dt, segs, ldx, ldg, W, perm, off, lr, opt, plan, plan_bytes, plan_id)
        else:
            need = ds.ds_group_sync_consensus_workspace_bytes(P, len(sizes))
            ws = torch.empty(need, dtype=torch.uint8, device=DEV)
            norms = torch.full((W,), -1.0, dtype=torch.float64, device=DEV)
            if tiled:
                ds.ds_group_sync_consensus_tiled(Xt, Gt, dt, P, tsx, tsg, W, perm, off, lr, norms, ws, need)
            else:
                ds.ds_group_sync_consensus(X, G, dt, P, ldx, ldg, W, perm, off, lr, norms, ws, need)
        torch.cuda.synchronize()
        runs = [(o, n) for o, n in segs if n] if layout == "ragged" else [(0, P)]
        for o, n in runs:
            oracle.step_opt(Xo, Go, perm, off, lr, V=Vo, momentum=mu, weight_decay=wd, S=So, factor=f, col0=o, ncols=n)
        if tiled:
            got = host(Xt, tsx)
            assert np.all(got[:, P:] == 7.0), case                  # unused slots of the last block
            got, got_v, got_s = got[:, :P], host(Vt, tsv)[:, :P] if use_v else None, host(St, tss)[:, :P] if use_s else None
        else:
            got = wl.tensor_to_numpy(X)
            touched = np.zeros(ldx, dtype=bool)
            for o, n in runs:
                touched[o:o + n] = True
            assert np.array_equal(got[:, ~touched], before[:, ~touched]), case   # padding, gaps between segments
            got_v, got_s = wl.tensor_to_numpy(V) if use_v else None, wl.tensor_to_numpy(S) if use_s else None
            if layout != "ragged":
                got, Xo = got[:, :P], Xo[:, :P]
                got_v, Vo = (got_v[:, :P], Vo[:, :P]) if use_v else (None, None)
                got_s, So = (got_s[:, :P], So[:, :P]) if use_s else (None, None)
        for a, b in ((got, Xo), (got_v, Vo), (got_s, So)):
            if a is not None:
                assert scaled_error(np.ascontiguousarray(a), np.ascontiguousarray(b)) <= TOL_F32, case
        if norms is not None:
            # the norms describe the state the GPU holds
            want = oracle.consensus(np.ascontiguousarray(got))
            if len(sizes) == 1:
                assert np.array_equal(norms.cpu().numpy(), np.zeros(W)), case
            else:
                np.testing.assert_allclose(norms.cpu().numpy(), want, rtol=1e-5, atol=1e-30, err_msg=case)
    if layout == "ragged":
        return
    need = ds.ds_consensus_workspace_bytes(W, P)
    ws, ws_g = (torch.empty(need, dtype=torch.uint8, device=DEV) for _ in range(2))
    full, grouped = (torch.full((W,), -1.0, dtype=torch.float64, device=DEV) for _ in range(2))
    if tiled:
        ds.ds_consensus_tiled(Xt, P, tsx, W, full, ws, need)
        ds.ds_consensus_grouped_tiled(Xt, P, tsx, W, perm, off, grouped, ws_g, need)
    else:
        ds.ds_consensus(X, P, ldx, W, full, ws, need)
        ds.ds_consensus_grouped(X, P, ldx, W, perm, off, grouped, ws_g, need)
    torch.cuda.synchronize()
    want = oracle.consensus(np.ascontiguousarray(got))
    np.testing.assert_allclose(full.cpu().numpy(), want, rtol=1e-5, atol=1e-30, err_msg=case)
    np.testing.assert_allclose(grouped.cpu().numpy(), want, rtol=1e-5, atol=1e-30, err_msg=case)
