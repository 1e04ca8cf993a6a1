"""Pins for the oracle's worker division (CPU only).

The division is integer work, so every check is exact: published splitmix64
outputs, golden permutations frozen with the shuffle's specification, a hand
trace for two workers done with Python integers, structure (Sec. IV-B2: the
groups are disjoint and cover every worker), counter-based behaviour and
uniformity of the shuffle.
"""
import numpy as np
import pytest

import oracle

MASK = 2**64 - 1


def test_splitmix64_published_outputs():
    # first three outputs of splitmix64 started from state 0 (public reference values)
    gamma = 0x9E3779B97F4A7C15
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    state = 0
    for w in want:
        state = (state + gamma) & MASK
        assert oracle.mix64(state) == w


def test_keys_golden(partition_golden):
    keys, _ = partition_golden
    for seed, t, want in keys:
        assert oracle.key(seed, t) == want


def test_permutations_golden(partition_golden):
    _, perms = partition_golden
    assert len(perms) >= 9
    for seed, t, W, want in perms:
        perm, off = oracle.partition(seed, t, W, [W])
        assert perm.tolist() == want
        assert off.tolist() == [0, W]


def test_two_workers_hand_trace():
    # W = 2 draws once; j = floor(r*2 / 2^64) is the top bit of r.  j == 1 leaves
    # the identity, j == 0 swaps.  Traced with Python integers; only mix64 (pinned
    # above against published values) is reused.
    gamma = 0x9E3779B97F4A7C15
    for seed, t in [(0, 0), (5, 17), (2**63 + 11, 2**40)]:
        s = oracle.mix64((oracle.mix64(seed) + (t + 1) * gamma) & MASK)
        r = oracle.mix64((s + gamma) & MASK)
        want = [0, 1] if (r >> 63) == 1 else [1, 0]
        perm, _ = oracle.partition(seed, t, 2, [1, 1])
        assert perm.tolist() == want


def test_three_workers_hand_trace():
    gamma = 0x9E3779B97F4A7C15
    for seed, t in [(0, 0), (9, 3), (77, 123456789)]:
        s = oracle.mix64((oracle.mix64(seed) + (t + 1) * gamma) & MASK)
        p = [0, 1, 2]
        s = (s + gamma) & MASK
        j = (oracle.mix64(s) * 3) >> 64
        p[2], p[j] = p[j], p[2]
        s = (s + gamma) & MASK
        j = (oracle.mix64(s) * 2) >> 64
        p[1], p[j] = p[j], p[1]
        perm, _ = oracle.partition(seed, t, 3, [2, 1])
        assert perm.tolist() == p


@pytest.mark.parametrize("W,sizes", [(1, [1]), (8, [4, 4]), (8, [2, 3, 3]), (16, [4] * 4),
                                     (32, [8] * 4), (64, [8] * 8), (7, [1, 1, 5]), (64, [64])])
def test_groups_are_a_disjoint_cover(W, sizes):
    for t in range(25):
        perm, off = oracle.partition(3, t, W, sizes)
        assert sorted(perm.tolist()) == list(range(W))
        assert off[0] == 0 and off[-1] == W
        assert np.diff(off).tolist() == list(sizes)


def test_counter_based_and_reseeded_every_iteration():
    a = [oracle.partition(11, t, 16, [4] * 4)[0].tolist() for t in range(30)]
    b = [oracle.partition(11, t, 16, [4] * 4)[0].tolist() for t in reversed(range(30))][::-1]
    assert a == b                      # order of calls is irrelevant
    assert len({tuple(p) for p in a}) > 25   # and iterations differ
    assert oracle.partition(12, 0, 16, [4] * 4)[0].tolist() != a[0]


def test_shuffle_is_uniform():
    # position of worker 0 and identity of perm[0] over many iterations: chi-square
    W, n = 8, 40000
    first = np.zeros(W)
    where0 = np.zeros(W)
    for t in range(n):
        perm, _ = oracle.partition(42, t, W, [W])
        first[perm[0]] += 1
        where0[int(np.where(perm == 0)[0][0])] += 1
    for counts in (first, where0):
        chi2 = float(((counts - n / W) ** 2 / (n / W)).sum())
        assert chi2 < 30.0             # 7 dof: P(chi2 > 30) ~ 1e-4


def test_rejects_bad_sizes():
    for W, sizes in [(8, [4, 3]), (8, [4, 4, 0]), (8, [9, -1]), (0, [])]:
        with pytest.raises(ValueError):
            oracle.partition(0, 0, W, sizes)
