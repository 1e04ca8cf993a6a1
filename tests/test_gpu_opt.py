"""GPU parity of the extended fused step (momentum, weight decay, SWA moving
average; Listing 1 and Sec. V-A3) against the CPU oracle, through the C ABI.
Same bars as the plain step: replica elements, momentum buffers and SWA models
within 1e-5 of max(|oracle|, rms(oracle row)); group members bit-identical."""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_03298_amd as ds
from paper_2007_03298_amd import workloads as wl
from test_gpu_parity import DEV, TOL_F32, assert_members_identical, random_stacks, scaled_error

pytestmark = pytest.mark.gpu

CASES = [
    # W, sizes, P, use V, use S, bf16 gradients
    (8, [4, 4], 3000, True, False, False),
    (8, [4, 4], 3001, False, True, False),
    (8, [2, 3, 3], 2563, True, True, False),
    (8, [8], 1027, True, True, True),
    (16, [5, 11], 777, True, True, False),
    (8, [1] * 8, 2049, True, True, False),
    (32, [8] * 4, 5003, True, True, False),
    (64, [64], 1030, True, True, False),
    (8, [4, 4], 2, True, True, False),
    (8, [4, 4], 4100, False, False, False),      # weight decay only
]


@pytest.mark.parametrize("W,sizes,P,use_v,use_s,bf16", CASES)
def test_extended_step_matches_oracle_small(W, sizes, P, use_v, use_s, bf16):
    ld = (P + 3) // 4 * 4
    ldv, lds = ld + 4, ld + 8                           # every stack with its own pitch
    X, G = random_stacks(300 + W + P, W, ld, ld, bf16)
    g = torch.Generator(device=DEV).manual_seed(5)
    V = torch.empty(W, ldv, dtype=torch.float32, device=DEV).normal_(generator=g) if use_v else None
    S = torch.empty(W, lds, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=g) if use_s else None
    Gh = wl.tensor_to_numpy(G)
    lr, mu, wd, f = 0.01, 0.9, 5e-4, 0.75
    opt = ds.local_opt(V, ldv, mu, wd, S, lds, f)
    for t in range(3):
        perm, off = ds.ds_partition(9, t, W, sizes)
        Xo = wl.tensor_to_numpy(X)
        Vo = wl.tensor_to_numpy(V) if use_v else None
        So = wl.tensor_to_numpy(S) if use_s else None
        v_pad = Vo[:, P:].copy() if use_v else None
        ds.ds_group_sync_opt(X, G, ds.DS_BF16 if bf16 else ds.DS_F32, P, ld, ld, W, perm, off, lr, opt)
        torch.cuda.synchronize()
        oracle.step_opt(Xo, Gh, perm, off, lr, V=Vo, momentum=mu, weight_decay=wd, S=So, factor=f, col0=0, ncols=P)
        got = wl.tensor_to_numpy(X)
        assert scaled_error(got[:, :P], Xo[:, :P]) <= TOL_F32
        assert_members_identical(got[:, :P], perm, off)
        if use_v:
            gv = wl.tensor_to_numpy(V)
            assert scaled_error(gv[:, :P], Vo[:, :P]) <= TOL_F32
            assert np.array_equal(gv[:, P:], v_pad)                    # padding untouched
        if use_s:
            assert scaled_error(wl.tensor_to_numpy(S)[:, :P], So[:, :P]) <= TOL_F32


def test_extended_step_without_state_is_the_plain_step():
    W, P, ld = 8, 5001, 5004
    X, G = random_stacks(71, W, ld, ld, False)
    X2 = X.clone()
    perm, off = ds.ds_partition(1, 0, W, [4, 4])
    ds.ds_group_sync(X, G, ds.DS_F32, P, ld, ld, W, perm, off, 0.01)
    ds.ds_group_sync_opt(X2, G, ds.DS_F32, P, ld, ld, W, perm, off, 0.01, ds.local_opt())
    X3 = X2.clone()
    ds.ds_group_sync_opt(X3, G, ds.DS_F32, P, ld, ld, W, perm, off, 0.0, None)
    torch.cuda.synchronize()
    assert torch.equal(X, X2)


def test_extended_step_ragged_bf16():
    W, sizes = 8, [4, 4]
    segs = [(0, 300), (320, 2047), (2368, 2049), (4424, 5), (4432, 0), (4480, 1025)]
    ld = 5512
    X, G = random_stacks(81, W, ld, ld, True)
    g = torch.Generator(device=DEV).manual_seed(6)
    V = torch.zeros(W, ld, dtype=torch.float32, device=DEV)
    S = X.clone()
    Gh = wl.tensor_to_numpy(G)
    nbytes = ds.ds_ragged_plan_bytes(segs)
    plan = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    plan_id = ds.ds_ragged_plan(segs, ld, ld, plan, nbytes)
    opt = ds.local_opt(V, ld, 0.9, 1e-3, S, ld, 0.5)
    for t in range(3):
        perm, off = ds.ds_partition(2, t, W, sizes)
        Xo, Vo, So = wl.tensor_to_numpy(X), wl.tensor_to_numpy(V), wl.tensor_to_numpy(S)
        before = (Xo.copy(), Vo.copy(), So.copy())
        ds.ds_group_sync_ragged_opt(X, G, ds.DS_BF16, segs, ld, ld, W, perm, off, 0.01, opt, plan, nbytes, plan_id)
        torch.cuda.synchronize()
        covered = np.zeros(ld, dtype=bool)
        for o, n in segs:
            oracle.step_opt(Xo, Gh, perm, off, 0.01, V=Vo, momentum=0.9, weight_decay=1e-3, S=So, factor=0.5,
                            col0=o, ncols=n)
            covered[o:o + n] = True
        for got_t, want, was in ((X, Xo, before[0]), (V, Vo, before[1]), (S, So, before[2])):
            got = wl.tensor_to_numpy(got_t)
            assert scaled_error(got[:, covered], want[:, covered]) <= TOL_F32
            assert np.array_equal(got[:, ~covered], was[:, ~covered])


def test_final_swa_average_is_one_group_of_all_workers():
    # Listing 1's last line: average the SWA models of all workers
    W, P, ld = 8, 4003, 4004
    S, _ = random_stacks(91, W, ld, ld, False)
    want = S[:, :P].double().mean(0).cpu().numpy()
    Z = torch.zeros_like(S)
    ds.ds_group_sync(S, Z, ds.DS_F32, P, ld, ld, W, list(range(W)), [0, W], 0.0)
    torch.cuda.synchronize()
    got = S[:, :P].cpu().numpy()
    assert scaled_error(got, np.tile(want, (W, 1)).astype(np.float32)) <= TOL_F32
    assert all(np.array_equal(got[0], got[i]) for i in range(W))


def test_config3_full_size_with_momentum_and_swa():
    from test_gpu_full_configs import Stage, pieces_of
    cfg = wl.CONFIGS[3]
    W, P = cfg.W, cfg.P
    ld = wl.padded_ld(P)
    free, _ = torch.cuda.mem_get_info()
    if free < 7 * W * ld * 4 + (3 << 30):
        pytest.skip("needs seven stacks of %.1f GB" % (W * ld * 4 / 1e9))
    run = wl.Run(cfg, DEV, P=P, ld=ld)
    X = run.init_params()
    V = torch.zeros_like(X)
    S = X.clone()
    G = torch.empty_like(X)
    rng = np.random.default_rng(33)
    cols = np.unique(np.concatenate([np.arange(0, 2048), np.arange(P - 2051, P)] +
                                    [np.arange(c, c + 300) for c in rng.integers(0, P - 300, 20)]))
    cols_t = torch.from_numpy(cols).to(DEV)
    Xo, Vo, So = (A.index_select(1, cols_t).cpu().numpy() for A in (X, V, S))
    opt = ds.local_opt(V, ld, 0.9, 5e-4, S, ld, 0.9)
    stage = Stage(W)
    for t in range(cfg.T):
        run.gradients(out=G)
        perm, off = ds.ds_partition(cfg.seed, t, W, cfg.sizes)
        last = t == cfg.T - 1
        if last:
            Xb, Vb, Sb = X.clone(), V.clone(), S.clone()
        Gw = G.index_select(1, cols_t).cpu().numpy()
        ds.ds_group_sync_opt(X, G, ds.DS_F32, P, ld, ld, W, perm, off, cfg.lr, opt)
        torch.cuda.synchronize()
        # trajectory on sampled windows: the oracle keeps its own X, V and S through all iterations
        oracle.step_opt(Xo, Gw, perm, off, cfg.lr, V=Vo, momentum=0.9, weight_decay=5e-4, S=So, factor=0.9)
        for A, want in ((X, Xo), (V, Vo), (S, So)):
            assert scaled_error(A.index_select(1, cols_t).cpu().numpy(), want) <= TOL_F32
    # the last iteration on EVERY column: oracle from the GPU's own pre-step state, all three stacks compared
    worst = 0.0
    for c0, n in pieces_of(0, P):
        xb, vb, sb = stage.pull("xb", Xb, c0, n), stage.pull("vb", Vb, c0, n), stage.pull("sb", Sb, c0, n)
        g = stage.pull("g", G, c0, n)
        xa, va, sa = stage.pull("xa", X, c0, n), stage.pull("va", V, c0, n), stage.pull("sa", S, c0, n)
        torch.cuda.synchronize()
        oracle.step_opt(xb, g, perm, off, cfg.lr, V=vb, momentum=0.9, weight_decay=5e-4, S=sb, factor=0.9)
        for got, want in ((xa, xb), (va, vb), (sa, sb)):
            err = oracle.scaled_error(got, want)
            assert err == err
            worst = max(worst, err)
    print("  extended step, all columns of X, V, S: %.2e" % worst, flush=True)
    assert worst <= TOL_F32
