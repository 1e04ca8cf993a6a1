"""Layer-by-layer synchronisation (Sec. V-A1: the backward hook of a layer
updates it locally and starts its group synchronisation without blocking, the
pre-forward hook waits for it; Sec. IV-A: L synchronisations per iteration)
against the CPU oracle, segment by segment.

One launch per layer, issued from the last layer to the first, round-robin on
K side streams that fork from the stream the gradients were produced on; one
event per layer.  The "next forward pass" is played by the main stream: it
waits for a layer's event and then reads that layer (a copy into a snapshot
buffer), with no device-wide synchronisation anywhere in between, so a
missing or misplaced wait shows up as stale values in the snapshot.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_03298_amd as ds
from paper_2007_03298_amd import workloads as wl
from test_gpu_parity import DEV, TOL_F32, assert_members_identical, scaled_error

pytestmark = pytest.mark.gpu

# a layer list with tiny, tile-sized, ragged and large layers (offsets on multiples of 8, gaps between them)
SEGS = [(0, 300), (320, 2047), (2368, 2049), (4424, 5), (4480, 1025), (5512, 70000), (75520, 300001), (375528, 1)]
LD = 375552


@pytest.mark.parametrize("extended", [False, True])
@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("K", [1, 2, 4])
def test_layer_by_layer_sync_matches_oracle(K, bf16, extended):
    W, sizes, lr, mu, wd, f = 8, [2, 3, 3], 0.01, 0.9, 5e-4, 0.75
    gen = torch.Generator(device=DEV).manual_seed(70 + K)
    X = torch.empty(W, LD, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=gen)
    G = torch.empty(W, LD, dtype=torch.bfloat16 if bf16 else torch.float32, device=DEV)
    V = torch.empty(W, LD, dtype=torch.float32, device=DEV).normal_(generator=gen) if extended else None
    S = X.clone() if extended else None
    snap = torch.zeros_like(X)
    lw = ds.LayerwiseSync(SEGS, K)
    covered = np.zeros(LD, dtype=bool)
    for o, n in SEGS:
        covered[o:o + n] = True
    Xo = wl.tensor_to_numpy(X)                        # the oracle keeps its own state through the iterations
    Vo = wl.tensor_to_numpy(V) if extended else None
    So = wl.tensor_to_numpy(S) if extended else None
    start = Xo.copy()
    kw = dict(V=V, ldv=LD, momentum=mu, weight_decay=wd, S=S, lds=LD, swa_factor=f) if extended else {}
    for t in range(3):
        perm, off = ds.ds_partition(12, t, W, sizes)
        # the gradients of this iteration are produced on the main stream right before the hooks fire
        G.copy_(torch.empty(W, LD, dtype=torch.float32, device=DEV).normal_(generator=gen))
        lw.backward(X, G, ds.DS_BF16 if bf16 else ds.DS_F32, LD, LD, W, perm, off, lr, **kw)
        # pre-forward hooks, first layer to last: wait for the layer, then use it
        for layer, (o, n) in enumerate(SEGS):
            lw.wait_layer(layer)
            snap[:, o:o + n].copy_(X[:, o:o + n])
        torch.cuda.synchronize()
        Gh = wl.tensor_to_numpy(G)
        for o, n in SEGS:
            if extended:
                oracle.step_opt(Xo, Gh, perm, off, lr, V=Vo, momentum=mu, weight_decay=wd, S=So, factor=f, col0=o, ncols=n)
            else:
                oracle.step(Xo, Gh, perm, off, lr, o, n)
        got = wl.tensor_to_numpy(snap)
        assert scaled_error(got[:, covered], Xo[:, covered]) <= TOL_F32
        assert_members_identical(got[:, covered], perm, off)
        assert np.array_equal(wl.tensor_to_numpy(X)[:, ~covered], start[:, ~covered])     # gaps never written
        if extended:
            assert scaled_error(wl.tensor_to_numpy(V)[:, covered], Vo[:, covered]) <= TOL_F32
            assert scaled_error(wl.tensor_to_numpy(S)[:, covered], So[:, covered]) <= TOL_F32
    assert not np.array_equal(Xo[:, covered], start[:, covered])


def test_layer_by_layer_wait_all_then_consensus_on_the_main_stream():
    # the whole-model use after all hooks: the consensus pass on the main stream sees every layer synchronised
    W, sizes, lr = 8, [4, 4], 0.02
    gen = torch.Generator(device=DEV).manual_seed(77)
    X = torch.empty(W, LD, dtype=torch.float32, device=DEV).normal_(0, 0.02, generator=gen)
    X[:, :] = X[0]                                         # identical models outside and inside the layers
    G = torch.empty(W, LD, dtype=torch.float32, device=DEV).normal_(generator=gen)
    lw = ds.LayerwiseSync(SEGS, 3)
    perm, off = ds.ds_partition(13, 0, W, sizes)
    Xo, Gh = wl.tensor_to_numpy(X), wl.tensor_to_numpy(G)
    need = ds.ds_consensus_workspace_bytes(W, LD)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = torch.zeros(W, dtype=torch.float64, device=DEV)
    lw.backward(X, G, ds.DS_F32, LD, LD, W, perm, off, lr)
    lw.wait_all()
    ds.ds_consensus(X, LD, LD, W, out, ws, need)
    torch.cuda.synchronize()
    for o, n in SEGS:
        oracle.step(Xo, Gh, perm, off, lr, o, n)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.consensus(Xo), rtol=1e-5)
