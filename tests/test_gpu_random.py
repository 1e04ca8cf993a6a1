"""Randomised GPU parity: random worker counts, divisions, column counts,
pitches, gradient types and optional state, each checked element by element
against the CPU oracle (same bars as the hand-picked cases)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_03298_amd as ds
from paper_2007_03298_amd import workloads as wl
from test_gpu_parity import DEV, TOL_F32, assert_members_identical, gpu_consensus, scaled_error

pytestmark = pytest.mark.gpu


def random_case(r):
    W = int(r.choice([1, 2, 3, 5, 8, 13, 16, 24, 32, 47, 64]))
    cuts = sorted(set(r.integers(1, W, size=int(r.integers(0, min(W, 7)))).tolist())) if W > 1 else []
    edges = [0] + cuts + [W]
    sizes = [b - a for a, b in zip(edges[:-1], edges[1:])]
    P = int(r.choice([1, 3, 4, 255, 256, 257, 1023, 1025, 2048, 2051, 4099, 9001, 20000]))
    pad = lambda n: (n + 3) // 4 * 4 + 4 * int(r.integers(0, 20))
    return W, sizes, P, pad(P), pad(P), pad(P), pad(P), bool(r.integers(0, 2)), bool(r.integers(0, 2)), bool(r.integers(0, 2))


@pytest.mark.parametrize("seed", range(40))
def test_random_case(seed):
    r = np.random.default_rng(5000 + seed)
    W, sizes, P, ldx, ldg, ldv, lds, bf16, use_v, use_s = random_case(r)
    g = torch.Generator(device=DEV).manual_seed(seed)
    X = torch.empty(W, ldx, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=g)
    G = torch.empty(W, ldg, dtype=torch.float32, device=DEV).normal_(generator=g)
    if bf16:
        G = G.to(torch.bfloat16)
    V = torch.empty(W, ldv, dtype=torch.float32, device=DEV).normal_(generator=g) if use_v else None
    S = torch.empty(W, lds, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=g) if use_s else None
    lr, mu, wd, f = float(r.choice([0.0, 0.01, 0.1])), 0.9, float(r.choice([0.0, 1e-3])), 0.8
    opt = ds.local_opt(V, ldv, mu, wd, S, lds, f)
    Gh = wl.tensor_to_numpy(G)
    for t in range(2):
        perm, off = ds.ds_partition(seed, t, W, sizes)
        Xo = wl.tensor_to_numpy(X)
        Vo = wl.tensor_to_numpy(V) if use_v else None
        So = wl.tensor_to_numpy(S) if use_s else None
        tail = Xo[:, P:].copy()
        ds.ds_group_sync_opt(X, G, ds.DS_BF16 if bf16 else ds.DS_F32, P, ldx, ldg, W, perm, off, lr, opt)
        torch.cuda.synchronize()
        oracle.step_opt(Xo, Gh, perm, off, lr, V=Vo, momentum=mu, weight_decay=wd, S=So, factor=f, col0=0, ncols=P)
        got = wl.tensor_to_numpy(X)
        assert scaled_error(got[:, :P], Xo[:, :P]) <= TOL_F32
        assert np.array_equal(got[:, P:], tail)
        assert_members_identical(got[:, :P], perm, off)
        if use_v:
            assert scaled_error(wl.tensor_to_numpy(V)[:, :P], Vo[:, :P]) <= TOL_F32
        if use_s:
            assert scaled_error(wl.tensor_to_numpy(S)[:, :P], So[:, :P]) <= TOL_F32
    d = gpu_consensus(X, P, ldx, W)
    want = oracle.consensus(wl.tensor_to_numpy(X), P)
    np.testing.assert_allclose(d, want, rtol=1e-5, atol=1e-30)
