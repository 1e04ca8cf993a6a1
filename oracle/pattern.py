"""Topology-aware divide-and-shuffle pattern (Sec. III-B) -- TEST INFRASTRUCTURE ONLY.

Plain-Python statement of how DS-Sync divides the workers of iteration t when
the rack of every worker is known, with the two adjustments the paper makes
for bandwidth contention.  The paper's figures for these patterns are not
available, so the rules below are a reading of its prose; where the prose
leaves a choice (which worker comes first in a rotation), the choice is stated.

Rules, in the paper's order:

* Static topology (Sec. III-B1).  The workers of a rack form an intra-rack
  group, except one representative per rack; the representatives form the
  inter-rack group.  The workers of a rack take turns as representative:
  in iteration t rack r sends ``eligible_r[t mod len(eligible_r)]`` (ascending
  worker index).  A rack therefore has exactly one worker, hence one
  connection, on its inter-rack link.
* Inter-rack link contention (Sec. III-B2).  The representative of every
  delayed rack is paired with one regular representative (a group of two);
  the remaining regular representatives form the large inter-rack group.
  The regular partner changes every iteration: the k-th delayed rack
  (ascending) takes regular rack ``regular[(t + k) mod len(regular)]``.
  If there are more delayed than regular racks, the delayed representatives
  left over are paired among themselves; if no rack is regular the flag makes
  no difference and all representatives form one group.
* End-host NIC contention (Sec. III-B3).  A delayed worker is never a
  representative.  If its rack has enough other workers, it is paired with
  one regular non-representative of the rack (a group of two), whose identity
  changes every iteration (``regular_nonreps[(t + k) mod len(...)]`` for the
  k-th delayed worker of the rack); the rest of the rack forms the large
  intra-rack group, the hub that exchanges members with the small group and
  with the inter-rack group.  "Enough" means at least one worker is left for
  the hub; otherwise the rack is not split.

Group order in the output: inter-rack pairs (delayed-rack order), the large
inter-rack group, then for every rack its small pairs and its large group.
"""
from __future__ import annotations

from math import gcd
from typing import List, Sequence, Tuple


def _racks(rack_of: Sequence[int]) -> List[List[int]]:
    n_racks = max(rack_of) + 1
    racks = [[] for _ in range(n_racks)]
    for w, r in enumerate(rack_of):
        if r < 0:
            raise ValueError("negative rack index")
        racks[r].append(w)
    if any(len(m) == 0 for m in racks):
        raise ValueError("every rack index below the largest must be used")
    return racks


def groups(rack_of: Sequence[int], slow_rack: Sequence[int], slow_worker: Sequence[int], t: int) -> List[List[int]]:
    """Groups of iteration t as lists of worker indices."""
    racks = _racks(rack_of)
    R = len(racks)
    if len(slow_rack) != R or len(slow_worker) != len(rack_of):
        raise ValueError("flag arrays do not match the topology")
    eligible = [[w for w in members if not slow_worker[w]] for members in racks]
    if any(len(e) == 0 for e in eligible):
        raise ValueError("a rack needs at least one worker without NIC contention")
    rep = [e[t % len(e)] for e in eligible]

    out: List[List[int]] = []
    if R >= 2:
        delayed = [r for r in range(R) if slow_rack[r]]
        regular = [r for r in range(R) if not slow_rack[r]]
        if not delayed or not regular:
            out.append(list(rep))
        else:
            taken = set()
            n_pairs = min(len(delayed), len(regular))
            for k in range(n_pairs):
                partner = regular[(t + k) % len(regular)]
                taken.add(partner)
                out.append([rep[delayed[k]], rep[partner]])
            rest = delayed[n_pairs:]
            for k in range(0, len(rest), 2):
                out.append([rep[r] for r in rest[k:k + 2]])
            large = [rep[r] for r in regular if r not in taken]
            if large:
                out.append(large)
    else:
        # a single rack has no inter-rack link: nobody is set apart
        rep = [None]

    for r, members in enumerate(racks):
        inside = [w for w in members if w != rep[r]]
        slow = [w for w in inside if slow_worker[w]]
        fast = [w for w in inside if not slow_worker[w]]
        if slow and len(fast) > len(slow):
            used = set()
            for k, z in enumerate(slow):
                q = fast[(t + k) % len(fast)]
                used.add(q)
                out.append([z, q])
            out.append([w for w in fast if w not in used])
        elif inside:
            out.append(inside)
    return out


def partition(rack_of, slow_rack, slow_worker, t) -> Tuple[List[int], List[int]]:
    """The same division as ``(perm, off)``: group k is ``perm[off[k]:off[k+1]]``."""
    perm: List[int] = []
    off = [0]
    for g in groups(rack_of, slow_rack, slow_worker, t):
        perm.extend(g)
        off.append(len(perm))
    return perm, off


def period(rack_of, slow_rack, slow_worker) -> int:
    """Number of iterations after which the pattern repeats (the paper's B)."""
    racks = _racks(rack_of)
    R = len(racks)
    lengths = []
    for members in racks:
        e = sum(1 for w in members if not slow_worker[w])
        if R >= 2:
            lengths.append(e)                       # turns as representative
        n_slow = len(members) - e
        n_fast_inside = e - (1 if R >= 2 else 0)
        if n_slow and n_fast_inside > n_slow:
            lengths.append(n_fast_inside)           # rotation of the small group's partner
    n_regular = sum(1 for r in range(R) if not slow_rack[r])
    if R >= 2 and 0 < n_regular < R:
        lengths.append(n_regular)                   # rotation of the regular partner
    B = 1
    for n in lengths:
        if n > 0:
            B = B * n // gcd(B, n)
    return B
