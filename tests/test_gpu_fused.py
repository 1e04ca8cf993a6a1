"""The step and the consensus norms of its result in one pass (``ds_group_sync_consensus``)
against the CPU oracle: replicas against ``oracle.step`` (and bit for bit
against ``ds_group_sync``), norms against ``oracle.consensus`` of the oracle's
own result."""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_03298_amd as ds
from paper_2007_03298_amd import workloads as wl
from test_gpu_parity import DEV, SMALL, TOL_F32, assert_members_identical, gpu_consensus, random_stacks, scaled_error

pytestmark = pytest.mark.gpu


def fused(X, G, dt, P, ldx, ldg, W, perm, off, lr):
    need = ds.ds_group_sync_consensus_workspace_bytes(P, len(off) - 1)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = torch.full((W,), -1.0, dtype=torch.float64, device=DEV)
    ds.ds_group_sync_consensus(X, G, dt, P, ldx, ldg, W, perm, off, lr, out, ws, need)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("W,sizes,P,ldx,ldg", SMALL + [(64, [4] * 16, 2100, None, None), (48, [1] * 47 + [1], 1000, None, None)])
def test_fused_step_and_norms_match_oracle_small(W, sizes, P, ldx, ldg, bf16):
    ldx = ldx or (P + 3) // 4 * 4
    ldg = ldg or (P + 3) // 4 * 4
    X, G = random_stacks(500 + W + P, W, ldx, ldg, bf16)
    Gh = wl.tensor_to_numpy(G)
    dt = ds.DS_BF16 if bf16 else ds.DS_F32
    for t in range(3):
        perm, off = ds.ds_partition(15, t, W, sizes)
        want = wl.tensor_to_numpy(X)
        twin = X.clone()
        d = fused(X, G, dt, P, ldx, ldg, W, perm, off, 0.01)
        ds.ds_group_sync(twin, G, dt, P, ldx, ldg, W, perm, off, 0.01)
        torch.cuda.synchronize()
        assert torch.equal(X, twin)                        # the same replicas as the plain step, bit for bit
        before = want.copy()
        oracle.step(want, Gh, perm, off, 0.01, 0, P)
        got = wl.tensor_to_numpy(X)
        assert scaled_error(got[:, :P], want[:, :P]) <= TOL_F32
        assert np.array_equal(got[:, P:], before[:, P:])
        assert_members_identical(got[:, :P], perm, off)
        d_want = oracle.consensus(want, P)
        if len(sizes) == 1:
            assert np.array_equal(d, np.zeros(W))          # one group: everybody holds the mean
        else:
            # the oracle's norms of its own result; tiny norms (a few columns) inherit the step's rounding
            np.testing.assert_allclose(d, d_want, rtol=1e-5 if P >= 64 else 1e-4)
            np.testing.assert_allclose(d, gpu_consensus(X, P, ldx, W), rtol=1e-6)
        for k in range(len(off) - 1):                      # members of a group share one norm
            assert len({d[i] for i in perm[off[k]:off[k + 1]]}) == 1


def test_fused_empty_input_writes_zero_norms():
    X, G = random_stacks(9, 8, 16, 16, False)
    before = X.clone()
    d = fused(X, G, ds.DS_F32, 0, 16, 16, 8, list(range(8)), [0, 4, 8], 0.01)
    assert torch.equal(X, before) and np.array_equal(d, np.zeros(8))


def test_fused_config1_trajectory():
    cfg = wl.CONFIGS[1]
    W, P = cfg.W, cfg.P
    ld = wl.padded_ld(P)
    run = wl.Run(cfg, DEV, P=P, ld=ld)
    X = run.init_params()
    Xo = wl.tensor_to_numpy(X)
    worst = 0.0
    for t in range(cfg.T):
        G = run.gradients()
        perm, off = ds.ds_partition(cfg.seed, t, W, cfg.sizes)
        d = fused(X, G, ds.DS_F32, P, ld, ld, W, perm, off, cfg.lr)
        oracle.step(Xo, wl.tensor_to_numpy(G), perm, off, cfg.lr, 0, P)
        worst = max(worst, scaled_error(wl.tensor_to_numpy(X)[:, :P], Xo[:, :P]))
        np.testing.assert_allclose(d, oracle.consensus(Xo, P), rtol=1e-5)
    assert worst <= TOL_F32


@pytest.mark.parametrize("idx", [2, 3])
def test_fused_full_size_against_the_two_pass_path(idx):
    # capped launches at benchmark size: replicas bit for bit those of ds_group_sync (itself held to the
    # oracle on every column elsewhere), norms against ds_consensus and the oracle on the whole stack
    from test_gpu_full_configs import Stage, oracle_consensus_streamed
    cfg = wl.CONFIGS[idx]
    W, P = cfg.W, cfg.P
    ld = wl.padded_ld(P)
    run = wl.Run(cfg, DEV, P=P, ld=ld)
    X = run.init_params()
    G = run.gradients()
    twin = X.clone()
    for t in range(2):
        perm, off = ds.ds_partition(cfg.seed, t, W, cfg.sizes)
        d = fused(X, G, ds.DS_F32, P, ld, ld, W, perm, off, cfg.lr)
        ds.ds_group_sync(twin, G, ds.DS_F32, P, ld, ld, W, perm, off, cfg.lr)
    torch.cuda.synchronize()
    assert torch.equal(X, twin)
    np.testing.assert_allclose(d, gpu_consensus(X, P, ld, W), rtol=1e-6)
    np.testing.assert_allclose(d, oracle_consensus_streamed(Stage(W), X, P), rtol=1e-5)
