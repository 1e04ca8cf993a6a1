"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.

Bars (fp32 replica arithmetic on the GPU, fp64 in the oracle):
  * worker division: bit exact;
  * members of a group after a step: bit identical;
  * replica elements: |gpu - oracle| <= 1e-5 * max(|oracle|, rms(oracle row))
    (2e-3 with bf16 gradients).  The denominator keeps the bound meaningful for
    elements near zero.  fp32 error budget per step: one rounding per local
    update, |g|-1 additions, one division -> about (|g|+2)/2 ulp of the
    largest partial sum, i.e. below 1e-6 of the row scale for |g| <= 64;
  * consensus norms: relative error <= 1e-5, exactly 0 for identical replicas.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_03298_amd as ds
from paper_2007_03298_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL_F32 = 1e-5
TOL_BF16 = 2e-3


def scaled_error(got: np.ndarray, want: np.ndarray) -> float:
    """max |got-want| / max(|want|, rms(want row)) over a [W, n] block."""
    want64 = want.astype(np.float64)
    rms = np.sqrt((want64**2).mean(axis=1, keepdims=True))
    den = np.maximum(np.abs(want64), np.maximum(rms, 1e-30))
    return float((np.abs(got.astype(np.float64) - want64) / den).max()) if want.size else 0.0


def assert_members_identical(Xh: np.ndarray, perm, off):
    bits = Xh.view(np.uint32)
    for k in range(len(off) - 1):
        members = perm[off[k]:off[k + 1]]
        for i in members[1:]:
            assert np.array_equal(bits[members[0]], bits[i])


def gpu_consensus(X: torch.Tensor, P: int, ld: int, W: int) -> np.ndarray:
    need = ds.ds_consensus_workspace_bytes(W, P)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = torch.full((W,), -1.0, dtype=torch.float64, device=DEV)
    ds.ds_consensus(X, P, ld, W, out, ws, need)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def random_stacks(seed, W, ldx, ldg, bf16):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    X = torch.empty(W, ldx, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=g)
    G = torch.empty(W, ldg, dtype=torch.float32, device=DEV).normal_(generator=g)
    if bf16:
        G = G.to(torch.bfloat16)
    return X, G


# ---------------------------------------------------------------- small, element by element

SMALL = [
    # W, sizes, P, ldx, ldg
    (8, [4, 4], 2048 * 3 + 517, None, None),          # several tiles and a ragged end
    (8, [2, 3, 3], 5000, 5004, 5008),                 # the paper's two-rack division, padded rows
    (8, [8], 4099, None, None),                       # one group: BSP
    (8, [1] * 8, 4097, None, None),                   # groups of one: independent SGD
    (5, [1, 4], 1, None, None),
    (3, [3], 2, None, None),
    (7, [3, 4], 3, None, None),
    (16, [4] * 4, 2047, None, None),
    (16, [5, 11], 2049, None, None),                  # more members than one round of loads
    (32, [8] * 4, 10000, None, None),
    (64, [8] * 8, 3000, None, None),
    (64, [64], 2500, None, None),
    (64, [1] * 63 + [1], 300, None, None),
    (1, [1], 777, None, None),
]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("W,sizes,P,ldx,ldg", SMALL)
def test_step_matches_oracle_small(W, sizes, P, ldx, ldg, bf16):
    ldx = ldx or (P + 3) // 4 * 4
    ldg = ldg or (P + 3) // 4 * 4
    X, G = random_stacks(100 + W + P, W, ldx, ldg, bf16)
    Xh0, Gh = wl.tensor_to_numpy(X), wl.tensor_to_numpy(G)
    for t in range(3):
        perm, off = ds.ds_partition(5, t, W, sizes)
        po, oo = oracle.partition(5, t, W, sizes)
        assert perm.tolist() == po.tolist() and off.tolist() == oo.tolist()
        before = wl.tensor_to_numpy(X)
        ds.ds_group_sync(X, G, ds.DS_BF16 if bf16 else ds.DS_F32, P, ldx, ldg, W, perm, off, 0.01)
        torch.cuda.synchronize()
        got = wl.tensor_to_numpy(X)
        want = before.copy()
        oracle.step(want, Gh, po, oo, 0.01, 0, P)
        assert scaled_error(got[:, :P], want[:, :P]) <= (TOL_BF16 if bf16 else TOL_F32)
        assert np.array_equal(got[:, P:], before[:, P:])          # padding columns untouched
        assert_members_identical(got[:, :P], perm, off)
    assert not np.array_equal(got[:, :P], Xh0[:, :P])


# Launches of more than one chip-load of workgroups are held to a number of
# wavefronts per CU that depends on the largest group, the gradient type and
# the momentum buffer; the small cases above never get there.
@pytest.mark.parametrize("W,sizes,bf16,use_v", [(8, [1, 2, 5], False, False), (8, [3, 5], True, False),
                                                (6, [1] * 6, False, False), (6, [2, 2, 2], True, True),
                                                (12, [1, 11], False, True), (4, [4], False, False)])
def test_occupancy_capped_launches_match_oracle(W, sizes, bf16, use_v):
    P = 256 * 8192 // len(sizes) + 256 * 700 + 77          # > 8192 workgroups, ragged end
    ld = ds.ds_padded_ld(P)
    X, G = random_stacks(31 + W, W, ld, ld, bf16)
    V = torch.empty_like(X).normal_(generator=torch.Generator(device=DEV).manual_seed(5)) if use_v else None
    Xh, Gh = wl.tensor_to_numpy(X), wl.tensor_to_numpy(G)
    Vh = wl.tensor_to_numpy(V) if use_v else None
    perm, off = ds.ds_partition(9, 4, W, sizes)
    if use_v:
        ds.ds_group_sync_opt(X, G, ds.DS_BF16 if bf16 else ds.DS_F32, P, ld, ld, W, perm, off, 0.02,
                             ds.local_opt(V, ld, 0.9, 1e-3, None, 0, 0.0))
        oracle.step_opt(Xh, Gh, perm, off, 0.02, V=Vh, momentum=0.9, weight_decay=1e-3, col0=0, ncols=P)
    else:
        ds.ds_group_sync(X, G, ds.DS_BF16 if bf16 else ds.DS_F32, P, ld, ld, W, perm, off, 0.02)
        oracle.step(Xh, Gh, perm, off, 0.02, 0, P)
    torch.cuda.synchronize()
    got = wl.tensor_to_numpy(X)
    assert scaled_error(got[:, :P], Xh[:, :P]) <= TOL_F32
    assert np.array_equal(got[:, P:], Xh[:, P:])
    assert_members_identical(got[:, :P], perm, off)
    if use_v:
        assert scaled_error(wl.tensor_to_numpy(V)[:, :P], Vh[:, :P]) <= TOL_F32


def test_group_of_all_workers_is_mean_gradient_sgd_on_gpu():
    W, P = 16, 6001
    ld = 6004
    X, G = random_stacks(7, W, ld, ld, False)
    xm = X[:, :P].double().mean(0)
    gm = G[:, :P].double().mean(0)
    perm, off = ds.ds_partition(0, 0, W, [W])
    ds.ds_group_sync(X, G, ds.DS_F32, P, ld, ld, W, perm, off, 0.05)
    torch.cuda.synchronize()
    want = (xm - float(np.float32(0.05)) * gm).cpu().numpy()
    got = X[:, :P].cpu().numpy()
    assert scaled_error(got, np.tile(want, (W, 1)).astype(np.float32)) <= TOL_F32
    assert np.array_equal(gpu_consensus(X, P, ld, W), np.zeros(W))


def test_bf16_path_equals_fp32_path_on_widened_gradients():
    W, P = 8, 9001
    ld = 9004
    X, G = random_stacks(8, W, ld, ld, True)
    X2 = X.clone()
    perm, off = ds.ds_partition(3, 1, W, [4, 4])
    ds.ds_group_sync(X, G, ds.DS_BF16, P, ld, ld, W, perm, off, 0.01)
    ds.ds_group_sync(X2, G.float(), ds.DS_F32, P, ld, ld, W, perm, off, 0.01)
    torch.cuda.synchronize()
    assert torch.equal(X, X2)          # widening is exact, so the two paths agree bit for bit


def test_empty_step_enqueues_nothing():
    X, G = random_stacks(9, 8, 16, 16, False)
    before = X.clone()
    ds.ds_group_sync(X, G, ds.DS_F32, 0, 16, 16, 8, list(range(8)), [0, 4, 8], 0.01)
    torch.cuda.synchronize()
    assert torch.equal(X, before)


# ---------------------------------------------------------------- ragged

def check_ragged(W, sizes, segs, ld, bf16, seed):
    X, G = random_stacks(seed, W, ld, ld, bf16)
    Gh = wl.tensor_to_numpy(G)
    nbytes = ds.ds_ragged_plan_bytes(segs)
    plan = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=DEV)
    plan_id = ds.ds_ragged_plan(segs, ld, ld, plan, nbytes)
    packed = ds.pack_segments(segs)
    for t in range(2):
        perm, off = ds.ds_partition(4, t, W, sizes)
        before = wl.tensor_to_numpy(X)
        ds.ds_group_sync_ragged(X, G, ds.DS_BF16 if bf16 else ds.DS_F32, packed, ld, ld, W, perm, off, 0.01,
                                plan, nbytes, plan_id)
        torch.cuda.synchronize()
        got = wl.tensor_to_numpy(X)
        want = before.copy()
        po, oo = oracle.partition(4, t, W, sizes)
        for o, n in segs:
            oracle.step(want, Gh, po, oo, 0.01, o, n)
        assert scaled_error(got, want) <= (TOL_BF16 if bf16 else TOL_F32)
        covered = np.zeros(ld, dtype=bool)
        for o, n in segs:
            covered[o:o + n] = True
        assert np.array_equal(got[:, ~covered], before[:, ~covered])   # gaps untouched
        assert_members_identical(got[:, covered], perm, off)


@pytest.mark.parametrize("bf16", [True, False])
def test_ragged_matches_oracle_small(bf16):
    segs = [(0, 256), (256, 1), (264, 0), (320, 2047), (2368, 2048), (4416, 2049), (6472, 7), (6528, 5000),
            (16384, 3), (16392, 1023), (17416, 1024), (18440, 1025), (19472, 255), (19728, 256), (19984, 257),
            (20248, 511), (20760, 512), (21272, 513)]
    check_ragged(8, [4, 4], segs, 21788, bf16, 21)
    check_ragged(8, [2, 3, 3], segs[::-1], 21788, bf16, 22)          # any order of the list
    check_ragged(8, [8], segs, 21788, bf16, 25)                      # a full round of eight members
    check_ragged(8, [2] * 4, segs, 21788, bf16, 26)                  # pairs
    check_ragged(8, [1] * 8, segs, 21788, bf16, 27)                  # groups of one
    check_ragged(32, [4] * 8, [(128 * i, 61 + i) for i in range(40)], 128 * 41, bf16, 23)


def test_ragged_equals_flat_on_one_segment():
    W, P, ld = 8, 50000, 50000
    X, G = random_stacks(24, W, ld, ld, True)
    X2 = X.clone()
    perm, off = ds.ds_partition(1, 1, W, [4, 4])
    segs = [(0, P)]
    nbytes = ds.ds_ragged_plan_bytes(segs)
    plan = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    plan_id = ds.ds_ragged_plan(segs, ld, ld, plan, nbytes)
    ds.ds_group_sync_ragged(X, G, ds.DS_BF16, segs, ld, ld, W, perm, off, 0.01, plan, nbytes, plan_id)
    ds.ds_group_sync(X2, G, ds.DS_BF16, P, ld, ld, W, perm, off, 0.01)
    torch.cuda.synchronize()
    assert torch.equal(X, X2)


def test_ragged_launch_tells_a_plan_of_another_list():
    W, ld = 8, 12288
    X, G = random_stacks(27, W, ld, ld, True)
    before = X.clone()
    perm, off = ds.ds_partition(1, 1, W, [4, 4])
    mine, other = [(0, 3000), (4096, 2000)], [(0, 2500), (4096, 1500)]       # same number of plan entries
    nbytes = ds.ds_ragged_plan_bytes(mine)
    assert nbytes == ds.ds_ragged_plan_bytes(other)
    plan = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    blank = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    plan_id = ds.ds_ragged_plan(mine, ld, ld, plan, nbytes)
    assert plan_id != 0 and plan_id == ds.ds_ragged_plan(mine, ld, ld, plan, nbytes)     # a function of the list
    # the host refuses a plan whose identity is not that of the list it is launched with
    with pytest.raises(ds.DsError) as e:
        ds.ds_group_sync_ragged(X, G, ds.DS_BF16, other, ld, ld, W, perm, off, 0.01, plan, nbytes, plan_id)
    assert e.value.status == -8
    # the device leaves the stacks alone when the buffer does not hold the plan it is told to expect
    ds.ds_group_sync_ragged(X, G, ds.DS_BF16, mine, ld, ld, W, perm, off, 0.01, blank, nbytes, plan_id)
    torch.cuda.synchronize()
    assert torch.equal(X, before)
    other_plan = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    other_id = ds.ds_ragged_plan(other, ld, ld, other_plan, nbytes)
    assert other_id != plan_id
    ds.ds_group_sync_ragged(X, G, ds.DS_BF16, mine, ld, ld, W, perm, off, 0.01, other_plan, nbytes, plan_id)
    torch.cuda.synchronize()
    assert torch.equal(X, before)
    # and the matching triple runs
    ds.ds_group_sync_ragged(X, G, ds.DS_BF16, mine, ld, ld, W, perm, off, 0.01, plan, nbytes, plan_id)
    torch.cuda.synchronize()
    want = wl.tensor_to_numpy(before)
    for o, n in mine:
        oracle.step(want, wl.tensor_to_numpy(G), perm, off, 0.01, o, n)
    assert scaled_error(wl.tensor_to_numpy(X), want) <= TOL_F32


def test_plan_of_many_segments_is_written_in_batches():
    # more segments than one launch of the plan kernel carries in its arguments
    W = 4
    segs = [(64 * i, 1 + (37 * i) % 64) for i in range(250)]
    ld = 64 * 250
    check_ragged(W, [2, 2], segs, ld, False, 28)


# ---------------------------------------------------------------- consensus

@pytest.mark.parametrize("W,P,ld", [(8, 1, 4), (8, 1023, 1024), (8, 100003, 100004), (5, 7777, 7780),
                                    (16, 50001, 50004), (13, 4096, 4096), (32, 30001, 30004),
                                    (33, 9999, 10000), (64, 20001, 20004), (1, 5000, 5000),
                                    (32, 2_100_000, 2_100_000)])
def test_consensus_matches_oracle(W, P, ld):
    X, _ = random_stacks(31 + W, W, ld, 4, False)
    got = gpu_consensus(X, P, ld, W)
    want = oracle.consensus(wl.tensor_to_numpy(X), P)
    if W == 1:
        assert np.array_equal(got, np.zeros(1))
    else:
        np.testing.assert_allclose(got, want, rtol=1e-5, atol=0)


def test_consensus_of_nearly_identical_replicas():
    # replicas that differ in the last bits only: the deviation is tiny against the
    # values, and must still be accurate relative to itself
    W, P = 8, 40000
    X, _ = random_stacks(41, 1, P, 4, False)
    X = X.repeat(W, 1).contiguous()
    Xi = X.view(torch.int32)
    bump = torch.randint(0, 3, (W, P), device=DEV, dtype=torch.int32,
                         generator=torch.Generator(device=DEV).manual_seed(1))
    Xi += bump
    got = gpu_consensus(X, P, P, W)
    want = oracle.consensus(wl.tensor_to_numpy(X), P)
    assert want.min() > 0
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=0)


def test_consensus_zero_for_identical_replicas_and_empty_input():
    for W in (3, 8, 24, 64):
        X, _ = random_stacks(51, 1, 5000, 4, False)
        X = X.repeat(W, 1).contiguous()
        assert np.array_equal(gpu_consensus(X, 5000, 5000, W), np.zeros(W))
    X, _ = random_stacks(52, 8, 16, 4, False)
    assert np.array_equal(gpu_consensus(X, 0, 16, 8), np.zeros(8))


def test_consensus_is_deterministic():
    X, _ = random_stacks(53, 32, 300000, 4, False)
    a = gpu_consensus(X, 300000, 300000, 32)
    b = gpu_consensus(X, 300000, 300000, 32)
    assert np.array_equal(a, b)


# ---------------------------------------------------------------- configuration 1: whole trajectory

def test_config1_trajectory_and_consensus():
    cfg = wl.CONFIGS[1]
    run = wl.Run(cfg, DEV)
    X = run.init_params()
    Xo = wl.tensor_to_numpy(X)                       # the oracle keeps its own state for all T
    assert np.array_equal(gpu_consensus(X, cfg.P, cfg.P, cfg.W), np.zeros(cfg.W))   # identical start
    worst_step, worst_traj = 0.0, 0.0
    for t in range(cfg.T):
        G = run.gradients()
        Gh = wl.tensor_to_numpy(G)
        perm, off = ds.ds_partition(cfg.seed, t, cfg.W, cfg.sizes)
        po, oo = oracle.partition(cfg.seed, t, cfg.W, cfg.sizes)
        assert perm.tolist() == po.tolist() and off.tolist() == oo.tolist()
        before = wl.tensor_to_numpy(X)
        ds.ds_group_sync(X, G, ds.DS_F32, cfg.P, cfg.P, cfg.P, cfg.W, perm, off, cfg.lr)
        torch.cuda.synchronize()
        got = wl.tensor_to_numpy(X)
        oracle.step(before, Gh, po, oo, cfg.lr)      # per step: oracle applied to the GPU's own state
        oracle.step(Xo, Gh, po, oo, cfg.lr)          # trajectory: oracle's own state
        worst_step = max(worst_step, scaled_error(got, before))
        worst_traj = max(worst_traj, scaled_error(got, Xo))
        assert_members_identical(got, perm, off)
        if t == 0:
            # closed-form expectation after the first step from identical models:
            # E d_i^2 = P lr^2 0.25 (1/|g| - 1/W)
            d = gpu_consensus(X, cfg.P, cfg.P, cfg.W)
            expect = np.sqrt(cfg.P * cfg.lr**2 * 0.25 * (1.0 / cfg.group - 1.0 / cfg.W))
            np.testing.assert_allclose(d, expect, rtol=0.01)
    assert worst_step <= TOL_F32 and worst_traj <= TOL_F32
    np.testing.assert_allclose(gpu_consensus(X, cfg.P, cfg.P, cfg.W), oracle.consensus(Xo), rtol=1e-5)


# ---------------------------------------------------------------- the paper's own pattern through the GPU path

def test_topology_pattern_drives_the_gpu_step():
    from oracle import mixing, pattern
    rack_of, slow_rack, slow_worker = [0, 0, 0, 0, 0, 1, 1, 1], [1, 0], [0, 0, 0, 0, 1, 0, 0, 0]
    W, P, ld = 8, 50001, 50004
    B = ds.ds_pattern_period(rack_of, slow_rack, slow_worker)
    X, G = random_stacks(61, W, ld, ld, False)
    Gh = wl.tensor_to_numpy(G)
    Xo = wl.tensor_to_numpy(X)
    for t in range(B):
        perm, off = ds.ds_pattern(rack_of, slow_rack, slow_worker, t)
        po, oo = pattern.partition(rack_of, slow_rack, slow_worker, t)
        assert perm.tolist() == po and off.tolist() == oo
        ds.ds_group_sync(X, G, ds.DS_F32, P, ld, ld, W, perm, off, 0.01)
        oracle.step(Xo, Gh, po, oo, 0.01, 0, P)
    torch.cuda.synchronize()
    got = wl.tensor_to_numpy(X)
    assert scaled_error(got[:, :P], Xo[:, :P]) <= TOL_F32
    # pure averaging over whole periods contracts the consensus norm as Lemma 1 bounds it
    mats = [mixing.mixing_matrix(*pattern.partition(rack_of, slow_rack, slow_worker, t)) for t in range(B)]
    sigma = mixing.contraction_norm(mixing.product(mats))
    assert sigma < 1.0
    fro2 = float((got[:, :P].astype(np.float64)**2).sum())
    Z = torch.zeros_like(G)
    for k in range(1, 4):
        for t in range(B):
            perm, off = ds.ds_pattern(rack_of, slow_rack, slow_worker, t)
            ds.ds_group_sync(X, Z, ds.DS_F32, P, ld, ld, W, perm, off, 0.0)
        d = gpu_consensus(X, P, ld, W)
        assert np.all(d**2 <= sigma**(2 * k) * fro2 * (1 + 1e-5) + 1e-9)


def test_layer_by_layer_launches_equal_the_ragged_launch():
    # Sec. V-A1: one synchronisation per layer; here one launch per segment on a view of the stacks
    W, sizes = 8, [4, 4]
    segs = [(0, 300), (320, 2047), (2368, 2049), (4424, 5), (4480, 1025), (5512, 70000)]
    ld = 75520
    X, G = random_stacks(95, W, ld, ld, True)
    X2 = X.clone()
    perm, off = ds.ds_partition(6, 0, W, sizes)
    nbytes = ds.ds_ragged_plan_bytes(segs)
    plan = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    plan_id = ds.ds_ragged_plan(segs, ld, ld, plan, nbytes)
    ds.ds_group_sync_ragged(X, G, ds.DS_BF16, segs, ld, ld, W, perm, off, 0.01, plan, nbytes, plan_id)
    streams = [torch.cuda.Stream() for _ in range(3)]
    torch.cuda.synchronize()
    for k, (o, n) in enumerate(reversed(segs)):
        ds.ds_group_sync(X2.data_ptr() + 4 * o, G.data_ptr() + 2 * o, ds.DS_BF16, n, ld, ld, W, perm, off, 0.01,
                         streams[k % 3])
    torch.cuda.synchronize()
    assert torch.equal(X, X2)


def gpu_consensus_grouped(X, P, ld, W, perm, off):
    need = ds.ds_consensus_workspace_bytes(W, P)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = torch.full((W,), -1.0, dtype=torch.float64, device=DEV)
    ds.ds_consensus_grouped(X, P, ld, W, perm, off, out, ws, need)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("W,sizes,P", [(8, [4, 4], 10001), (8, [2, 3, 3], 4097), (32, [8] * 4, 300001),
                                      (64, [8] * 8, 20003), (64, [1] * 64, 5000), (16, [16], 3000),
                                      (33, [11, 22], 1027)])
def test_grouped_consensus_after_a_step(W, sizes, P):
    # right after a step the members of a group are identical: one row per group is enough
    ld = (P + 3) // 4 * 4
    X, G = random_stacks(400 + W, W, ld, ld, False)
    perm, off = ds.ds_partition(8, 3, W, sizes)
    ds.ds_group_sync(X, G, ds.DS_F32, P, ld, ld, W, perm, off, 0.01)
    got = gpu_consensus_grouped(X, P, ld, W, perm, off)
    full = gpu_consensus(X, P, ld, W)
    want = oracle.consensus(wl.tensor_to_numpy(X), P)
    if len(sizes) == 1:
        assert np.array_equal(got, np.zeros(W))
    else:
        np.testing.assert_allclose(got, want, rtol=1e-5)
        np.testing.assert_allclose(got, full, rtol=1e-6)
    # members of a group share one value
    for k in range(len(off) - 1):
        assert len({got[i] for i in perm[off[k]:off[k + 1]]}) == 1


def test_grouped_consensus_describes_the_first_members_when_rows_differ():
    # the documented behaviour off the precondition: every member counts as its group's first member
    W, P, ld = 8, 3001, 3004
    X, _ = random_stacks(450, W, ld, 4, False)
    perm, off = ds.ds_partition(2, 0, W, [4, 4])
    got = gpu_consensus_grouped(X, P, ld, W, perm, off)
    Xr = wl.tensor_to_numpy(X).copy()
    for k in range(2):
        for i in perm[off[k]:off[k + 1]]:
            Xr[i] = Xr[perm[off[k]]]
    np.testing.assert_allclose(got, oracle.consensus(Xr, P), rtol=1e-5)
