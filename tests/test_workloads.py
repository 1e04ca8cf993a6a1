"""The input side (no arithmetic of the method): the configuration table, the
row pitch, the ragged layer list and the layout conversion the tiled tests
rely on."""
import numpy as np
import torch

import paper_2007_03298_amd as ds
from paper_2007_03298_amd import workloads as wl


def test_configurations_are_the_five_named_ones():
    c = wl.CONFIGS
    assert [c[i].W for i in (1, 2, 3, 4, 5)] == [8, 16, 32, 64, 32]
    assert [c[i].group for i in (1, 2, 3, 4, 5)] == [4, 4, 8, 8, 4]
    assert [c[i].P for i in (1, 2, 3, 4)] == [1048576, 11689512, 25557032, 138357544]
    assert [c[i].T for i in (1, 2, 3, 4, 5)] == [20, 10, 5, 3, 5]
    assert [c[i].seed for i in (1, 2, 3, 4, 5)] == [0, 1, 2, 3, 4]
    assert c[4].lr == 0.005 and all(c[i].lr == 0.01 for i in (1, 2, 3, 5))
    assert c[5].ragged and c[5].bf16_grads and c[3].worker_scale and not c[4].worker_scale
    for i in (1, 2, 3, 4, 5):
        assert sum(c[i].sizes) == c[i].W and set(c[i].sizes) == {c[i].group}


def test_padded_pitch_agrees_with_the_library():
    for P in (1, 255, 256, 257, 1048576, 11689512, 25557032, 138357544):
        ld = wl.padded_ld(P)
        assert ld == ds.ds_padded_ld(P) and ld >= P and ld % 256 == 0 and (ld // 256) % 2 == 1 and ld - P < 512


def test_ragged_layer_list_of_configuration_5():
    segs, ld, attempt = wl.ragged_segments(wl.CONFIGS[5].seed)
    lengths = [n for _, n in segs]
    assert len(segs) == 199 and attempt == 0 and sum(lengths) == 100519676 and ld == 100545792
    assert min(lengths) >= 256 and max(lengths) <= 4194304
    assert max(lengths) / min(lengths) > 1000                       # spans orders of magnitude
    ends = 0
    for o, n in segs:                                               # in order, disjoint, on multiples of 256 elements
        assert o % 256 == 0 and o >= ends
        ends = o + n
    assert ends <= ld
    assert wl.ragged_segments(wl.CONFIGS[5].seed)[0] == segs        # deterministic


def test_tiled_layout_conversion():
    rng = np.random.default_rng(0)
    for W, P, slack in ((5, 1, 0), (8, 256, 0), (8, 1000, 512), (32, 2563, 256), (3, 70001, 0)):
        ld = (P + 3) // 4 * 4 + 8
        rows = torch.from_numpy(rng.standard_normal((W, ld)).astype(np.float32))
        ts = W * 256 + slack
        t = wl.to_tiled(rows, P, ts)
        n_tiles = (P + 255) // 256
        assert t.numel() == n_tiles * ts and n_tiles * W * 256 == ds.ds_tiled_elements(P, W)
        # element (i, p) at (p // 256) * tile_stride + i * 256 + p % 256
        for i, p in ((0, 0), (W - 1, P - 1), (W // 2, P // 2), (W - 1, min(P - 1, 255)), (0, max(P - 256, 0))):
            assert t[(p // 256) * ts + i * 256 + p % 256] == rows[i, p]
        back = wl.from_tiled(t, P, W, ts)
        assert back.shape == (W, n_tiles * 256) and torch.equal(back[:, :P], rows[:, :P])
        assert torch.all(back[:, P:] == 7.0)                        # slots that stand for no column
        if slack:
            assert torch.all(t.view(n_tiles, ts)[:, W * 256:] == 7.0)
    bits = torch.from_numpy(rng.standard_normal((4, 520)).astype(np.float32)).to(torch.bfloat16)
    assert torch.equal(wl.from_tiled(wl.to_tiled(bits, 513), 513, 4)[:, :513], bits[:, :513])
