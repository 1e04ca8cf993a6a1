"""Pins for the topology-aware divide-and-shuffle pattern (CPU only).

The paper's figures of these patterns are missing, so the pins are the
statements its prose makes (Sec. III-B1..3, Sec. IV-B2) and the worker layouts
of its three testbed scenarios (Sec. V-A5): a valid division every iteration;
one worker per rack on the inter-rack link; everyone takes turns as
representative; a delayed rack's representative sits in a group of two whose
regular partner changes every iteration; a worker with NIC contention never
leaves its rack and sits in a group of two; the pattern is periodic and its
period product is connected (second eigenvalue below one), so pure averaging
with the oracle's step contracts as Lemma 1 says.
"""
import numpy as np
import pytest

import oracle
from oracle import mixing, pattern


def check_valid(groups, W):
    flat = [w for g in groups for w in g]
    assert sorted(flat) == list(range(W))
    assert all(len(g) >= 1 for g in groups)


def inter_rack_groups(groups, rack_of):
    return [g for g in groups if len({rack_of[w] for w in g}) > 1]


SCENARIO_STATIC = dict(rack_of=[0, 0, 0, 0, 1, 1, 1, 1], slow_rack=[0, 0], slow_worker=[0] * 8)
SCENARIO_LINK = dict(rack_of=[0, 0, 0, 0, 1, 1, 1, 1], slow_rack=[1, 0], slow_worker=[0] * 8)
SCENARIO_NIC = dict(rack_of=[0, 0, 0, 0, 0, 1, 1, 1], slow_rack=[1, 0], slow_worker=[0, 0, 0, 0, 1, 0, 0, 0])
FOUR_RACKS = dict(rack_of=[r for r in range(4) for _ in range(4)], slow_rack=[0, 0, 0, 0], slow_worker=[0] * 16)
FOUR_RACKS_LINK = dict(rack_of=[r for r in range(4) for _ in range(4)], slow_rack=[1, 0, 0, 0], slow_worker=[0] * 16)


def test_static_two_racks_is_one_inter_and_two_intra_groups():
    # the static scenario of the testbed: one inter-rack group and two intra-rack groups
    topo = SCENARIO_STATIC
    reps_seen = set()
    for t in range(8):
        gs = pattern.groups(t=t, **topo)
        check_valid(gs, 8)
        assert sorted(len(g) for g in gs) == [2, 3, 3]
        inter = inter_rack_groups(gs, topo["rack_of"])
        assert len(inter) == 1 and sorted(topo["rack_of"][w] for w in inter[0]) == [0, 1]
        reps_seen.update(inter[0])
        for g in gs:
            if g is not inter[0]:
                assert len({topo["rack_of"][w] for w in g}) == 1
    assert reps_seen == set(range(8))          # everybody takes a turn within one period
    assert pattern.period(**topo) == 4


def test_four_racks_static_and_with_a_delayed_link():
    for t in range(8):
        gs = pattern.groups(t=t, **FOUR_RACKS)
        check_valid(gs, 16)
        assert sorted(len(g) for g in gs) == [3, 3, 3, 3, 4]
    partners = []
    for t in range(6):
        gs = pattern.groups(t=t, **FOUR_RACKS_LINK)
        check_valid(gs, 16)
        assert sorted(len(g) for g in gs) == [2, 2, 3, 3, 3, 3]
        inter = inter_rack_groups(gs, FOUR_RACKS_LINK["rack_of"])
        assert len(inter) == 2
        small = [g for g in inter if 0 in {FOUR_RACKS_LINK["rack_of"][w] for w in g}]
        assert len(small) == 1 and len(small[0]) == 2      # the delayed rack is in the smallest group
        partner_rack = [FOUR_RACKS_LINK["rack_of"][w] for w in small[0] if FOUR_RACKS_LINK["rack_of"][w] != 0][0]
        partners.append(partner_rack)
        # every rack still has exactly one worker on its inter-rack link
        on_link = [FOUR_RACKS_LINK["rack_of"][w] for g in inter for w in g]
        assert sorted(on_link) == [0, 1, 2, 3]
    assert all(a != b for a, b in zip(partners, partners[1:]))   # the regular partner changes every iteration
    assert set(partners) == {1, 2, 3}


def test_nic_contention_keeps_the_delayed_worker_inside_its_rack_in_a_pair():
    topo = SCENARIO_NIC
    partners = []
    for t in range(12):
        gs = pattern.groups(t=t, **topo)
        check_valid(gs, 8)
        mine = [g for g in gs if 4 in g][0]
        assert len(mine) == 2
        other = [w for w in mine if w != 4][0]
        assert topo["rack_of"][other] == 0 and other != 4
        partners.append(other)
        inter = inter_rack_groups(gs, topo["rack_of"])
        assert all(4 not in g for g in inter)              # never a representative
        assert sorted(len(g) for g in gs) == [2, 2, 2, 2]
    assert all(a != b for a, b in zip(partners, partners[1:]))
    assert set(partners) == {0, 1, 2, 3}
    B = pattern.period(**topo)
    assert B == 12
    for t in range(B):
        assert pattern.groups(t=t, **topo) == pattern.groups(t=t + B, **topo)


def test_degenerate_topologies():
    one_rack = dict(rack_of=[0] * 5, slow_rack=[0], slow_worker=[0] * 5)
    assert pattern.groups(t=3, **one_rack) == [[0, 1, 2, 3, 4]]        # no inter-rack link: plain BSP
    singles = dict(rack_of=[0, 1, 2], slow_rack=[0, 0, 0], slow_worker=[0, 0, 0])
    assert pattern.groups(t=5, **singles) == [[0, 1, 2]]
    all_slow_racks = dict(rack_of=[0, 0, 1, 1], slow_rack=[1, 1], slow_worker=[0] * 4)
    assert sorted(len(g) for g in pattern.groups(t=0, **all_slow_racks)) == [1, 1, 2]
    with pytest.raises(ValueError):
        pattern.groups([0, 0, 1], [0, 0], [0, 0, 1], 0)               # rack 1 has only a delayed worker
    with pytest.raises(ValueError):
        pattern.groups([0, 2], [0, 0, 0], [0, 0], 0)                  # rack 1 is empty


@pytest.mark.parametrize("topo", [SCENARIO_STATIC, SCENARIO_LINK, SCENARIO_NIC, FOUR_RACKS, FOUR_RACKS_LINK])
def test_period_product_is_connected_and_averaging_contracts(topo):
    W = len(topo["rack_of"])
    B = pattern.period(**topo)
    mats = []
    for t in range(B):
        perm, off = pattern.partition(t=t, **topo)
        assert pattern.partition(t=t + B, **topo) == (perm, off)
        M = mixing.mixing_matrix(perm, off)
        np.testing.assert_allclose(M.sum(0), 1.0)
        mats.append(M)
    P_B = mixing.product(mats)
    rho = mixing.second_eigenvalue(P_B)
    sigma = mixing.contraction_norm(P_B)
    assert rho < 1.0 - 1e-6 and sigma < 1.0 - 1e-6        # all workers exchange information within a period
    # pure averaging with the oracle's step: the consensus norm shrinks as Lemma 1 bounds it
    X = np.random.default_rng(3).standard_normal((W, 40)).astype(np.float32)
    fro2 = float((X.astype(np.float64)**2).sum())
    Z = np.zeros_like(X)
    for k in range(1, 5):
        for t in range(B):
            perm, off = pattern.partition(t=t, **topo)
            oracle.step(X, Z, perm, off, 0.0)
        d = oracle.consensus(X)
        assert np.all(d**2 <= sigma**(2 * k) * fro2 + 1e-9)


def test_random_topologies_are_always_valid_and_periodic():
    r = np.random.default_rng(11)
    for _ in range(300):
        R = int(r.integers(1, 6))
        sizes = r.integers(1, 7, size=R)
        rack_of = [k for k in range(R) for _ in range(int(sizes[k]))]
        W = len(rack_of)
        slow_rack = (r.random(R) < 0.3).astype(int).tolist()
        slow_worker = (r.random(W) < 0.2).astype(int).tolist()
        for k in range(R):                      # keep one worker per rack free of NIC contention
            members = [w for w in range(W) if rack_of[w] == k]
            if all(slow_worker[w] for w in members):
                slow_worker[members[0]] = 0
        B = pattern.period(rack_of, slow_rack, slow_worker)
        for t in range(min(B, 40)):
            gs = pattern.groups(rack_of, slow_rack, slow_worker, t)
            check_valid(gs, W)
            inter = inter_rack_groups(gs, rack_of)
            on_link = [rack_of[w] for g in inter for w in g]
            assert len(on_link) == len(set(on_link))        # at most one worker per rack crosses racks
            assert all(not slow_worker[w] for g in inter for w in g)
            assert gs == pattern.groups(rack_of, slow_rack, slow_worker, t + B)
