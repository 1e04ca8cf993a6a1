"""Host-side checks of libdssync.so that need no GPU: the library loads, exports
every symbol the header declares, its worker division agrees bit for bit with
the oracle's independent implementation, and every argument error is reported
before anything touches a device."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2007_03298_amd as ds
from paper_2007_03298_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dssync.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ds_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_header_is_c99_and_a_plain_c_client_links_and_runs(tmp_path, partition_golden):
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    exe = str(tmp_path / "abi_client")
    libdir = os.path.dirname(binding.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "abi_client.c"), "-L", libdir, "-l:libdssync.so",
                    "-Wl,-rpath," + libdir, "-o", exe], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, (res.returncode, res.stdout, res.stderr)
    want = [p for s, t, W, p in partition_golden[1] if (s, t, W) == (0, 0, 8)][0]
    assert res.stdout.split("perm")[1].split() == [str(v) for v in want]


def test_status_strings():
    for code in range(0, -10, -1):
        s = ds.status_string(code)
        assert s.startswith("DS_")
    assert not ds.status_string(-99).startswith("DS_")


def test_padded_ld_is_the_smallest_odd_multiple_of_256_that_holds_the_row():
    from paper_2007_03298_amd import workloads as wl
    r = np.random.default_rng(5)
    cases = [0, 1, 255, 256, 257, 511, 512, 513, 1_048_576, 11_689_512, 25_557_032, 138_357_544]
    cases += [int(v) for v in r.integers(0, 2**40, size=2000)]
    for P in cases:
        ld = ds.ds_padded_ld(P)
        assert ld >= P and ld % 256 == 0 and (ld // 256) % 2 == 1
        assert ld - P < 512                      # at most one pad unit beyond the plain round-up
        smaller = ld - 512                       # the next odd multiple below does not hold the row
        assert smaller < P
        assert ld == wl.padded_ld(P)             # the benchmark layout is the library's recommendation
    assert ds.ds_padded_ld(-1) == 0
    assert ds.ds_padded_ld(2**63 - 1) == 0


def test_partition_golden(partition_golden):
    _, perms = partition_golden
    for seed, t, W, want in perms:
        perm, off = ds.ds_partition(seed, t, W, [W])
        assert perm.tolist() == want and off.tolist() == [0, W]


def test_partition_bit_exact_against_oracle_on_random_inputs():
    r = np.random.default_rng(2024)
    for _ in range(10000):
        W = int(r.integers(1, ds.DS_MAX_W + 1))
        # random composition of W into groups
        cuts = sorted(set(r.integers(1, W, size=int(r.integers(0, min(W, 9)))).tolist())) if W > 1 else []
        edges = [0] + cuts + [W]
        sizes = [b - a for a, b in zip(edges[:-1], edges[1:])]
        seed = int(r.integers(0, 2**63)) * 2 + int(r.integers(0, 2))
        t = int(r.integers(0, 2**63)) if r.random() < 0.2 else int(r.integers(0, 100000))
        p1, o1 = ds.ds_partition(seed, t, W, sizes)
        p2, o2 = oracle.partition(seed, t, W, sizes)
        assert p1.tolist() == p2.tolist() and o1.tolist() == o2.tolist()


def test_partition_errors():
    def status(*a):
        with pytest.raises(ds.DsError) as e:
            ds.ds_partition(*a)
        return e.value.status
    assert status(0, 0, 0, [1]) == -2
    assert status(0, 0, ds.DS_MAX_W + 1, [ds.DS_MAX_W + 1]) == -2
    assert status(0, 0, 8, [4, 3]) == -3
    assert status(0, 0, 8, [8, 0]) == -3
    assert status(0, 0, 8, [9, -1]) == -3
    assert status(0, 0, 8, []) == -3
    lib = ctypes.CDLL(binding.LIB_PATH)
    lib.ds_partition.restype = ctypes.c_int
    assert lib.ds_partition(ctypes.c_uint64(0), ctypes.c_uint64(0), 4, None, 1, None, None) == -1


# ---- argument validation of the GPU entry points (nothing is launched) ----------

A = 4096          # a 16-byte aligned stand-in address; never dereferenced because
B = 1 << 20       # every call below must fail validation first
PERM8 = list(range(8))
OFF8 = [0, 4, 8]


def sync_status(X=A, G=B, dt=0, P=16, ldx=16, ldg=16, W=8, perm=PERM8, off=OFF8):
    with pytest.raises(ds.DsError) as e:
        ds.ds_group_sync(X, G, dt, P, ldx, ldg, W, perm, off, 0.1, stream=0)
    return e.value.status


def test_group_sync_argument_errors():
    assert sync_status(X=0) == -1
    assert sync_status(G=0) == -1
    assert sync_status(dt=2) == -7
    assert sync_status(P=-1) == -5
    assert sync_status(P=20) == -5                  # ld < P
    assert sync_status(ldx=18, P=10) == -6          # ld not a multiple of 4
    assert sync_status(X=A + 4) == -6
    assert sync_status(G=B + 8) == -6
    assert sync_status(W=0, perm=[], off=[0]) == -2
    assert sync_status(W=65, perm=list(range(65)), off=[0, 65]) == -2
    assert sync_status(perm=[0, 1, 2, 3, 4, 5, 6, 6]) == -4
    assert sync_status(perm=[0, 1, 2, 3, 4, 5, 6, 8]) == -4
    assert sync_status(off=[0, 4, 7]) == -4
    assert sync_status(off=[0, 4, 4, 8]) == -4      # empty group
    assert sync_status(off=[1, 4, 8]) == -4


def test_rows_longer_than_one_launch_covers_are_refused_before_any_device_call():
    # gridDim.x * 64 threads must stay below 2^32: 2^26 - 1 tiles of 256 columns
    assert ds.DS_MAX_COLUMNS == (2**26 - 1) * 256
    too_long = ds.DS_MAX_COLUMNS + 4
    assert sync_status(P=too_long, ldx=too_long, ldg=too_long, W=1, perm=[0], off=[0, 1]) == -5
    assert sync_status(P=2**40, ldx=2**40, ldg=2**40) == -5
    need = ds.ds_consensus_workspace_bytes(8, 100)
    with pytest.raises(ds.DsError) as e:
        ds.ds_consensus(A, too_long, too_long, 8, B, 3 * B, need, stream=0)
    assert e.value.status == -5


def test_group_sync_empty_is_ok_without_a_device():
    ds.ds_group_sync(A, B, 0, 0, 16, 16, 8, PERM8, OFF8, 0.1, stream=0)   # P == 0: nothing enqueued


def ragged_status(segs, X=A, G=B, ldx=4096, ldg=4096, plan=A, plan_bytes=1 << 20, plan_id=1):
    with pytest.raises(ds.DsError) as e:
        ds.ds_group_sync_ragged(X, G, 1, segs, ldx, ldg, 8, PERM8, OFF8, 0.1, plan, plan_bytes, plan_id, stream=0)
    return e.value.status


def test_ragged_argument_errors():
    assert ragged_status([(4, 16)]) == -6           # offset not a multiple of 8
    assert ragged_status([(0, -1)]) == -5
    assert ragged_status([(-8, 4)]) == -5
    assert ragged_status([(4000, 200)]) == -5       # runs past the leading dimension
    assert ragged_status([(0, 16)], plan=0) == -8
    assert ragged_status([(0, 16)], plan_bytes=8) == -8
    assert ragged_status([(0, 16)], plan=A + 8) == -8
    assert ragged_status([(0, 16)], plan_bytes=16) == -8       # room for the header only
    # a plan that was not built from this list: its identity is not the list's, whatever it is
    for wrong in (0, 1, 12345, 2**64 - 1):
        assert ragged_status([(0, 16), (64, 100)], plan_id=wrong) == -8
    # one launch covers at most DS_MAX_COLUMNS columns, of a ragged list too
    huge = ds.DS_MAX_COLUMNS + 2048
    assert ragged_status([(0, huge)], ldx=huge, ldg=huge) == -5
    # all-empty segment lists enqueue nothing and need no plan
    ds.ds_group_sync_ragged(A, B, 1, [(0, 0), (64, 0)], 4096, 4096, 8, PERM8, OFF8, 0.1, 0, 0, 0, stream=0)
    ds.ds_group_sync_ragged(A, B, 1, [], 4096, 4096, 8, PERM8, OFF8, 0.1, 0, 0, 0, stream=0)


def test_ragged_plan_bytes_and_plan_errors():
    assert ds.ds_ragged_plan_bytes([]) == 0
    assert ds.ds_ragged_plan_bytes([(0, 0)]) == 0
    one = ds.ds_ragged_plan_bytes([(0, 1)])
    assert one == 32                                 # a header entry and one tile entry, 16 bytes each
    # the tile width is the library's business, but the entry count is additive
    # over segments and grows with the length
    a, b, c = (0, 100000), (100096, 7), (200000, 12345)
    entries = lambda segs: ds.ds_ragged_plan_bytes(segs) // 16 - 1
    assert entries([a, b, c]) == sum(entries([x]) for x in (a, b, c))
    assert entries([b]) == 1
    assert entries([a]) > entries([c]) > 1
    assert ds.ds_ragged_plan_bytes([a]) % 16 == 0
    assert ds.ds_ragged_plan_bytes([(3, 5)]) == 0   # invalid list
    with pytest.raises(ds.DsError) as e:
        ds.ds_ragged_plan([(0, 64), (32, 64)], 4096, 4096, A, 1 << 20, stream=0)   # overlap
    assert e.value.status == -5
    with pytest.raises(ds.DsError) as e:
        ds.ds_ragged_plan([(0, 64)], 4096, 4096, A, 16, stream=0)
    assert e.value.status == -8
    assert ds.ds_ragged_plan([(0, 0)], 4096, 4096, 0, 0, stream=0) == 0   # nothing to build: identity 0
    lib = ctypes.CDLL(binding.LIB_PATH)
    seg = binding.ds_segment(0, 64)
    assert lib.ds_ragged_plan(ctypes.byref(seg), 1, ctypes.c_int64(64), ctypes.c_int64(64), ctypes.c_void_p(A),
                              ctypes.c_size_t(64), None, None) == -1        # nowhere to put the identity


def test_consensus_argument_errors():
    need = ds.ds_consensus_workspace_bytes(8, 100)
    assert need > 0 and need % 16 == 0
    assert ds.ds_consensus_workspace_bytes(0, 100) == 0
    assert ds.ds_consensus_workspace_bytes(65, 100) == 0

    def status(X=A, P=16, ld=16, W=8, out=B, ws=3 * B, ws_bytes=need):
        with pytest.raises(ds.DsError) as e:
            ds.ds_consensus(X, P, ld, W, out, ws, ws_bytes, stream=0)
        return e.value.status
    assert status(X=0) == -1
    assert status(out=0) == -1
    assert status(W=0) == -2
    assert status(W=65) == -2
    assert status(P=-1) == -5
    assert status(P=17) == -5
    assert status(ld=18, P=10) == -6
    assert status(X=A + 4) == -6
    assert status(out=B + 4) == -6
    assert status(ws=0) == -8
    assert status(ws_bytes=need - 1) == -8
    assert status(ws=3 * B + 8) == -8


def test_fused_step_and_consensus_argument_errors():
    need = ds.ds_group_sync_consensus_workspace_bytes(16, 2)
    assert need >= 16 and ds.ds_group_sync_consensus_workspace_bytes(1000, 3) == 4 * 3 * 8
    assert ds.ds_group_sync_consensus_workspace_bytes(-1, 2) == 0
    assert ds.ds_group_sync_consensus_workspace_bytes(16, 0) == 0
    assert ds.ds_group_sync_consensus_workspace_bytes(ds.DS_MAX_COLUMNS + 4, 2) == 0

    def status(X=A, G=B, P=16, ld=16, W=8, perm=PERM8, off=OFF8, out=2 * B, ws=3 * B, ws_bytes=need):
        with pytest.raises(ds.DsError) as e:
            ds.ds_group_sync_consensus(X, G, 0, P, ld, ld, W, perm, off, 0.1, out, ws, ws_bytes, stream=0)
        return e.value.status
    assert status(X=0) == -1
    assert status(out=0) == -1
    assert status(out=2 * B + 4) == -6
    assert status(P=17) == -5
    assert status(perm=[0, 1, 2, 3, 4, 5, 6, 6]) == -4
    assert status(ws=0) == -8
    assert status(ws=3 * B + 8) == -8
    assert status(ws_bytes=need - 1) == -8


def test_static_scratch_consensus_checks_its_arguments_like_the_workspace_one():
    lib = ctypes.CDLL(binding.LIB_PATH)
    lib.ds_consensus_static.restype = ctypes.c_int
    lib.ds_consensus_static.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                        ctypes.c_void_p, ctypes.c_void_p]
    assert lib.ds_consensus_static(None, 16, 16, 8, B, None) == -1
    assert lib.ds_consensus_static(A, 16, 16, 8, None, None) == -1
    assert lib.ds_consensus_static(A, 16, 16, 65, B, None) == -2          # beyond its array: more than DS_MAX_W workers
    assert lib.ds_consensus_static(A, 16, 16, 0, B, None) == -2
    assert lib.ds_consensus_static(A, 17, 16, 8, B, None) == -5
    assert lib.ds_consensus_static(A, ds.DS_MAX_COLUMNS + 4, 2**40, 8, B, None) == -5   # beyond one launch
    assert lib.ds_consensus_static(A + 4, 16, 16, 8, B, None) == -6
    assert lib.ds_consensus_static(A, 16, 16, 8, B + 4, None) == -6


# ---- topology-aware pattern: library against the oracle's independent implementation ----

def random_topology(r):
    R = int(r.integers(1, 7))
    sizes = r.integers(1, 9, size=R)
    rack_of = [k for k in range(R) for _ in range(int(sizes[k]))]
    W = len(rack_of)
    slow_rack = (r.random(R) < 0.3).astype(int).tolist()
    slow_worker = (r.random(W) < 0.25).astype(int).tolist()
    for k in range(R):
        members = [w for w in range(W) if rack_of[w] == k]
        if all(slow_worker[w] for w in members):
            slow_worker[members[int(r.integers(0, len(members)))]] = 0
    order = r.permutation(W)                     # workers of a rack need not be contiguous
    return [rack_of[i] for i in order], slow_rack, [slow_worker[i] for i in order]


def test_pattern_bit_exact_against_oracle_on_random_topologies():
    from oracle import pattern
    r = np.random.default_rng(77)
    for _ in range(2000):
        rack_of, slow_rack, slow_worker = random_topology(r)
        B = ds.ds_pattern_period(rack_of, slow_rack, slow_worker)
        assert B == pattern.period(rack_of, slow_rack, slow_worker)
        for t in [0, 1, 2, int(r.integers(0, 1000)), B, int(r.integers(0, 2**62))]:
            perm, off = ds.ds_pattern(rack_of, slow_rack, slow_worker, t)
            p2, o2 = pattern.partition(rack_of, slow_rack, slow_worker, t)
            assert perm.tolist() == p2 and off.tolist() == o2


def test_pattern_check_against_dense_mixing_matrices():
    # Sec. IV-B2: connectivity of one period and the contraction factors of its product, against
    # numpy on the dense matrices (eigenvalues of the product; 2-norm of its non-consensus part)
    from oracle import mixing, pattern
    r = np.random.default_rng(78)
    seen_disconnected = 0
    for trial in range(300):
        if trial % 3 == 0:
            # an arbitrary periodic list of random divisions (often not connected when short)
            W = int(r.integers(1, 20))
            divisions = []
            for _ in range(int(r.integers(1, 4))):
                cuts = sorted(set(r.integers(1, W, size=int(r.integers(0, W))).tolist())) if W > 1 else []
                edges = [0] + cuts + [W]
                divisions.append((r.permutation(W).tolist(), edges))
        else:
            rack_of, slow_rack, slow_worker = random_topology(r)
            W = len(rack_of)
            Bp = min(pattern.period(rack_of, slow_rack, slow_worker), 60)
            divisions = [pattern.partition(rack_of, slow_rack, slow_worker, t) for t in range(Bp)]
        connected, rho, sigma = ds.ds_pattern_check(W, divisions)
        M = mixing.product([mixing.mixing_matrix(p, o) for p, o in divisions])
        want_rho = mixing.second_eigenvalue(M) if W > 1 else 0.0
        want_sigma = mixing.contraction_norm(M)
        # components of the union graph, by brute force: boolean closure of the summed adjacency
        reach = sum(mixing.mixing_matrix(p, o) for p, o in divisions) > 0
        for _ in range(7):                       # paths of up to 2^7 >= DS_MAX_W edges
            reach = (reach.astype(np.int64) @ reach.astype(np.int64)) > 0
        want_connected = bool(reach.all())
        assert connected == want_connected
        assert abs(rho - want_rho) <= 1e-7 * max(1.0, want_rho) + 1e-9, (trial, rho, want_rho)
        assert abs(sigma - want_sigma) <= 1e-9
        assert (rho < 1 - 1e-9) == connected and (sigma < 1 - 1e-9) == connected
        assert rho <= sigma + 1e-12
        seen_disconnected += not connected
    assert 10 < seen_disconnected < 290
    # the testbed layouts of Sec. V-A5 are connected over a period; one iteration of them is not
    static = ([0, 0, 0, 0, 1, 1, 1, 1], [0, 0], [0] * 8)
    period = [tuple(a.tolist() for a in ds.ds_pattern(*static, t)) for t in range(ds.ds_pattern_period(*static))]
    assert ds.ds_pattern_check(8, period)[0] and not ds.ds_pattern_check(8, period[:1])[0]
    # a single group of everyone reaches consensus in one step
    assert ds.ds_pattern_check(5, [(list(range(5)), [0, 5])]) == (True, 0.0, 0.0)


def test_pattern_check_errors():
    lib = ctypes.CDLL(binding.LIB_PATH)
    i32 = lambda v: (ctypes.c_int32 * len(v))(*v)
    out = ctypes.c_int32(7)
    call = lambda W, Bn, perm, off, n: lib.ds_pattern_check(W, Bn, i32(perm), i32(off), i32(n), ctypes.byref(out), None, None)
    assert call(4, 1, [0, 1, 2, 3], [0, 2, 4, 0, 0], [2]) == 0 and out.value == 0
    assert call(0, 1, [0], [0, 0], [1]) == -2
    assert call(4, 0, [0, 1, 2, 3], [0, 2, 4, 0, 0], [2]) == -5
    assert call(4, 1, [0, 1, 2, 2], [0, 2, 4, 0, 0], [2]) == -4
    assert call(4, 1, [0, 1, 2, 3], [0, 2, 3, 0, 0], [2]) == -4
    assert call(4, 1, [0, 1, 2, 3], [0, 2, 4, 0, 0], [0]) == -3
    assert lib.ds_pattern_check(4, 1, None, i32([0, 4]), i32([1]), ctypes.byref(out), None, None) == -1


def test_pattern_testbed_layouts():
    # the three worker layouts of the paper's testbed (Sec. V-A5)
    static = ([0, 0, 0, 0, 1, 1, 1, 1], [0, 0], [0] * 8)
    nic = ([0, 0, 0, 0, 0, 1, 1, 1], [1, 0], [0, 0, 0, 0, 1, 0, 0, 0])
    for t in range(8):
        perm, off = ds.ds_pattern(*static, t)
        assert sorted(np.diff(off).tolist()) == [2, 3, 3]
        assert perm[:2].tolist() == [t % 4, 4 + t % 4]
        perm, off = ds.ds_pattern(*nic, t)
        assert sorted(np.diff(off).tolist()) == [2, 2, 2, 2]
    assert ds.ds_pattern_period(*static) == 4
    assert ds.ds_pattern_period(*nic) == 12


def test_pattern_errors():
    def status(*a):
        with pytest.raises(ds.DsError) as e:
            ds.ds_pattern(*a)
        return e.value.status
    assert status([0, 0, 1], [0, 0], [0, 0, 1], 0) == -10        # rack 1 has only a delayed worker
    assert status([0, 2], [0, 0, 0], [0, 0], 0) == -10           # rack 1 unused
    assert status([0, 3], [0, 0], [0, 0], 0) == -10              # rack index out of range
    assert status([0, -1], [0, 0], [0, 0], 0) == -10
    assert status([], [0], [], 0) == -2
    assert status([0] * 65, [0], [0] * 65, 0) == -2
    with pytest.raises(ds.DsError) as e:
        ds.ds_pattern_period([0, 2], [0, 0, 0], [0, 0])
    assert e.value.status == -10


def test_extended_step_argument_errors():
    def status(opt, P=16, ld=16):
        with pytest.raises(ds.DsError) as e:
            ds.ds_group_sync_opt(A, B, 0, P, ld, ld, 8, PERM8, OFF8, 0.1, opt, stream=0)
        return e.value.status
    assert status(ds.local_opt(V=2 * B + 4, ldv=16)) == -6           # misaligned buffer
    assert status(ds.local_opt(V=2 * B, ldv=18)) == -6               # pitch not a multiple of 4
    assert status(ds.local_opt(V=2 * B, ldv=12)) == -5               # pitch below P
    assert status(ds.local_opt(S=2 * B, lds=8)) == -5
    assert status(ds.local_opt(S=2 * B + 8, lds=16)) == -6
    # nothing to do: P == 0 succeeds without a device
    ds.ds_group_sync_opt(A, B, 0, 0, 16, 16, 8, PERM8, OFF8, 0.1, ds.local_opt(V=2 * B, ldv=16), stream=0)
    with pytest.raises(ds.DsError) as e:
        ds.ds_group_sync_ragged_opt(A, B, 1, [(0, 64)], 4096, 4096, 8, PERM8, OFF8, 0.1,
                                    ds.local_opt(V=2 * B, ldv=32), A, 1 << 20, 1, stream=0)
    assert e.value.status == -5                                      # buffer pitch ends before the segment


def test_grouped_consensus_argument_errors():
    need = ds.ds_consensus_workspace_bytes(8, 100)

    def status(perm=PERM8, off=OFF8, **kw):
        args = dict(X=A, P=16, ld=16, W=8, out=B, ws=3 * B, ws_bytes=need)
        args.update(kw)
        with pytest.raises(ds.DsError) as e:
            ds.ds_consensus_grouped(args["X"], args["P"], args["ld"], args["W"], perm, off, args["out"], args["ws"],
                                    args["ws_bytes"], stream=0)
        return e.value.status
    assert status(X=0) == -1
    assert status(P=17) == -5
    assert status(ws_bytes=need - 1) == -8
    assert status(perm=[0, 1, 2, 3, 4, 5, 6, 6]) == -4
    assert status(off=[0, 4, 7]) == -4


def test_tiled_entry_points_check_their_arguments():
    # ds_tiled_elements: whole blocks of W * 256 elements
    assert ds.ds_tiled_elements(1000, 8) == 4 * 8 * 256
    assert ds.ds_tiled_elements(0, 8) == 0 and ds.ds_tiled_elements(256, 64) == 64 * 256
    assert ds.ds_tiled_elements(-1, 8) == 0 and ds.ds_tiled_elements(10, 0) == 0 and ds.ds_tiled_elements(10, 65) == 0
    assert ds.ds_tiled_elements(ds.DS_MAX_COLUMNS + 4, 1) == 0
    block = 8 * 256

    def step(X=A, G=B, dt=0, P=1000, tsx=block, tsg=block, W=8, perm=PERM8, off=OFF8, opt=None):
        with pytest.raises(ds.DsError) as e:
            ds.ds_group_sync_tiled(X, G, dt, P, tsx, tsg, W, perm, off, 0.1, opt, stream=0)
        return e.value.status
    assert step(X=0) == -1 and step(G=0) == -1
    assert step(dt=3) == -7
    assert step(P=-1) == -5
    assert step(tsx=block - 256) == -5              # blocks would overlap
    assert step(tsg=block - 256) == -5
    assert step(tsx=block + 4) == -6                # blocks start on whole tiles
    assert step(X=A + 8) == -6
    assert step(W=0, perm=[], off=[0]) == -2
    assert step(off=[0, 4, 4, 8]) == -4
    assert step(opt=ds.local_opt(V=3 * B, ldv=block - 256, momentum=0.9)) == -5
    assert step(opt=ds.local_opt(S=3 * B, lds=block + 4, swa_factor=0.5)) == -6
    # the 1-D grid holds tiles * groups workgroups
    many = ds.DS_MAX_COLUMNS // 4 + 256
    assert step(P=many, W=8, perm=PERM8, off=list(range(9))) == -5
    ds.ds_group_sync_tiled(A, B, 0, 0, block, block, 8, PERM8, OFF8, 0.1, stream=0)     # P == 0: nothing enqueued

    need = ds.ds_consensus_workspace_bytes(8, 1000)
    def cons(X=A, P=1000, ts=block, W=8, out=2 * B, ws=3 * B, ws_bytes=need):
        with pytest.raises(ds.DsError) as e:
            ds.ds_consensus_tiled(X, P, ts, W, out, ws, ws_bytes, stream=0)
        return e.value.status
    assert cons(X=0) == -1 and cons(out=0) == -1
    assert cons(ts=block - 256) == -5
    assert cons(ts=block + 8) == -6
    assert cons(W=65) == -2
    assert cons(ws=0) == -8 and cons(ws_bytes=need - 1) == -8

    def grouped(X=A, ts=block, off=OFF8, ws_bytes=need):
        with pytest.raises(ds.DsError) as e:
            ds.ds_consensus_grouped_tiled(X, 1000, ts, 8, PERM8, off, 2 * B, 3 * B, ws_bytes, stream=0)
        return e.value.status
    assert grouped(X=0) == -1
    assert grouped(ts=block - 256) == -5 and grouped(ts=block + 8) == -6
    assert grouped(off=[0, 4, 7]) == -4
    assert grouped(ws_bytes=need - 1) == -8

    need2 = ds.ds_group_sync_consensus_workspace_bytes(1000, 2)
    def fused(X=A, P=1000, tsx=block, out=2 * B, ws=3 * B, ws_bytes=need2, off=OFF8):
        with pytest.raises(ds.DsError) as e:
            ds.ds_group_sync_consensus_tiled(X, B, 0, P, tsx, block, 8, PERM8, off, 0.1, out, ws, ws_bytes, stream=0)
        return e.value.status
    assert fused(X=0) == -1 and fused(out=0) == -1
    assert fused(tsx=block - 256) == -5
    assert fused(off=[0, 4, 7]) == -4
    assert fused(ws_bytes=need2 - 1) == -8
