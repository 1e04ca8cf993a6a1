"""Pins for the oracle's synchronisation step and consensus norm (CPU only).

Each test checks ``ds_oracle.c`` against something that is not itself: dense
mixing-matrix products (Sec. IV-B2), the closed-form trajectory (Sec. III-A
step 4), textbook special cases computed with numpy (group size N is
single-machine SGD on the mean gradient, Sec. I; group size 1 is independent
SGD), invariants of a doubly stochastic matrix, Lemma 1's bound with the
eigenvalues from numpy, and a closed-form expectation.
"""
import numpy as np
import pytest

import oracle
from oracle import mixing


def rng_stack(seed, W, P, scale=1.0):
    r = np.random.default_rng(seed)
    return (scale * r.standard_normal((W, P))).astype(np.float32)


def rack_pattern(k):
    """Static-topology division of Sec. III-B1 for the 8-worker, 2-rack testbed
    (workers 0-3 and 4-7, Sec. V-A5): one representative per rack forms the
    inter-rack group, the rest of each rack stays intra-rack, and the workers
    of a rack take turns as representative.  Sizes {2, 3, 3}, period 4."""
    r0, r1 = k % 4, 4 + k % 4
    perm = [r0, r1] + [w for w in range(4) if w != r0] + [w for w in range(4, 8) if w != r1]
    return np.array(perm, dtype=np.int32), np.array([0, 2, 5, 8], dtype=np.int32)


DIVISIONS = [
    (8, [4, 4]), (8, [2, 3, 3]), (8, [8]), (8, [1] * 8), (6, [1, 2, 3]), (5, [5]), (7, [3, 4]),
]


@pytest.mark.parametrize("W,sizes", DIVISIONS)
def test_step_equals_dense_mixing_matrix(W, sizes):
    P = 37
    for t in range(4):
        X = rng_stack(10 + t, W, P, 0.02)
        G = rng_stack(20 + t, W, P)
        perm, off = oracle.partition(7, t, W, sizes)
        want = mixing.step_dense(X, G, perm, off, 0.01)
        got = X.copy()
        oracle.step(got, G, perm, off, 0.01)
        # the only difference allowed is the final rounding to fp32 (one ulp where
        # the two fp64 summation orders straddle a rounding boundary)
        np.testing.assert_allclose(got, want.astype(np.float32), rtol=2.0**-23, atol=1e-45)


def test_mixing_matrix_is_symmetric_doubly_stochastic():
    for W, sizes in DIVISIONS:
        perm, off = oracle.partition(1, 5, W, sizes)
        M = mixing.mixing_matrix(perm, off)
        assert np.array_equal(M, M.T)
        assert np.all(M >= 0)
        np.testing.assert_allclose(M.sum(0), 1.0, atol=1e-15)
        np.testing.assert_allclose(M.sum(1), 1.0, atol=1e-15)
        vals = set(np.unique(M).tolist())
        assert vals <= {0.0} | {1.0 / s for s in sizes}


def test_pure_averaging_trajectory_is_the_matrix_product():
    # no gradients: X_K = W_{K-1} ... W_0 X_0, later divisions on the left
    W, P, T = 8, 16, 6
    X0 = rng_stack(3, W, P)
    Z = np.zeros((W, P), dtype=np.float32)
    X = X0.copy()
    mats = []
    for t in range(T):
        perm, off = oracle.partition(5, t, W, [2, 3, 3])
        mats.append(mixing.mixing_matrix(perm, off))
        oracle.step(X, Z, perm, off, 0.01)
    want = mixing.product(mats) @ X0.astype(np.float64)
    # fp32 storage between iterations: one rounding per iteration
    np.testing.assert_allclose(X, want, rtol=0, atol=T * 2.0**-24 * np.abs(X0).max())
    # and the order matters: the reversed product is a different matrix
    rev = mixing.product(mats[::-1]) @ X0.astype(np.float64)
    assert np.abs(rev - want).max() > 1e-3


def test_trajectory_matches_closed_form():
    # identical initial models, local updates Delta_t = -lr * G_t
    W, P, T, lr = 8, 24, 5, 0.01
    x0 = (0.02 * np.random.default_rng(0).standard_normal(P)).astype(np.float32)
    X = np.tile(x0, (W, 1))
    mats, deltas = [], []
    for t in range(T):
        G = rng_stack(100 + t, W, P)
        perm, off = oracle.partition(9, t, W, [4, 4])
        mats.append(mixing.mixing_matrix(perm, off))
        deltas.append(-float(np.float32(lr)) * G.astype(np.float64))
        oracle.step(X, G, perm, off, lr)
    want = mixing.closed_form(x0, deltas, mats)
    np.testing.assert_allclose(X, want, rtol=0, atol=T * 2.0**-24 * np.abs(want).max())


def test_one_group_of_all_workers_is_single_machine_sgd():
    W, P, lr = 16, 101, 0.05
    X = rng_stack(1, W, P, 0.02)
    G = rng_stack(2, W, P)
    perm, off = oracle.partition(0, 0, W, [W])
    got = X.copy()
    oracle.step(got, G, perm, off, lr)
    lr32 = float(np.float32(lr))
    want = X.astype(np.float64).mean(0) - lr32 * G.astype(np.float64).mean(0)
    for i in range(W):
        np.testing.assert_allclose(got[i], want, rtol=2.0**-23, atol=0)
    assert all(np.array_equal(got[0], got[i]) for i in range(W))
    np.testing.assert_array_equal(oracle.consensus(got), np.zeros(W))


def test_groups_of_one_are_independent_sgd():
    W, P, lr = 5, 33, 0.01
    X = rng_stack(4, W, P)
    G = rng_stack(5, W, P)
    perm, off = oracle.partition(0, 3, W, [1] * W)
    got = X.copy()
    oracle.step(got, G, perm, off, lr)
    want = (X.astype(np.float64) - float(np.float32(lr)) * G.astype(np.float64)).astype(np.float32)
    np.testing.assert_array_equal(got, want)


def test_groups_do_not_interact():
    W, P = 8, 40
    X = rng_stack(6, W, P)
    G = rng_stack(7, W, P)
    perm, off = oracle.partition(2, 2, W, [4, 4])
    a = X.copy()
    oracle.step(a, G, perm, off, 0.01)
    X2, G2 = X.copy(), G.copy()
    X2[perm[:4]] += 3.0          # disturb group 0 only
    G2[perm[:4]] *= -2.0
    b = X2.copy()
    oracle.step(b, G2, perm, off, 0.01)
    np.testing.assert_array_equal(a[perm[4:]], b[perm[4:]])
    assert not np.array_equal(a[perm[:4]], b[perm[:4]])


def test_global_mean_is_preserved_and_members_are_identical():
    W, P = 8, 64
    X = rng_stack(8, W, P, 0.02)
    G = rng_stack(9, W, P)
    perm, off = oracle.partition(4, 1, W, [2, 3, 3])
    Y = X.astype(np.float64) - float(np.float32(0.01)) * G.astype(np.float64)
    got = X.copy()
    oracle.step(got, G, perm, off, 0.01)
    np.testing.assert_allclose(got.astype(np.float64).mean(0), Y.mean(0), rtol=0,
                               atol=2.0**-24 * np.abs(Y).max())
    for members in mixing.groups_of(perm, off):
        for i in members[1:]:
            assert np.array_equal(got[members[0]].view(np.uint32), got[i].view(np.uint32))


def test_zero_lr_averaging_is_idempotent_and_identical_rows_are_a_fixed_point():
    W, P = 8, 20
    X = rng_stack(11, W, P)
    G = rng_stack(12, W, P)
    perm, off = oracle.partition(1, 1, W, [4, 4])
    a = X.copy()
    oracle.step(a, G, perm, off, 0.0)
    b = a.copy()
    oracle.step(b, G, perm, off, 0.0)
    np.testing.assert_array_equal(a, b)
    same = np.tile(X[0], (W, 1))
    c = same.copy()
    oracle.step(c, np.zeros_like(G), perm, off, 0.3)
    np.testing.assert_array_equal(c, same)


def test_column_window_and_leading_dimensions():
    W, P, ldx, ldg = 4, 10, 16, 12
    X = rng_stack(13, W, ldx)
    G = rng_stack(14, W, ldg)
    perm, off = oracle.partition(0, 0, W, [2, 2])
    got = X.copy()
    oracle.step(got, G, perm, off, 0.01, col0=2, ncols=7)
    want = mixing.step_dense(X[:, 2:9], G[:, 2:9], perm, off, 0.01).astype(np.float32)
    np.testing.assert_array_equal(got[:, 2:9], want)
    np.testing.assert_array_equal(got[:, :2], X[:, :2])
    np.testing.assert_array_equal(got[:, 9:], X[:, 9:])


def test_bf16_gradients_are_widened_exactly():
    W, P = 8, 50
    X = rng_stack(15, W, P, 0.02)
    G32 = rng_stack(16, W, P)
    bits = (G32.view(np.uint32) >> 16).astype(np.uint16)        # some bf16 values
    widened = (bits.astype(np.uint32) << 16).view(np.float32)
    perm, off = oracle.partition(4, 0, W, [4, 4])
    a, b = X.copy(), X.copy()
    oracle.step(a, bits, perm, off, 0.01)
    oracle.step(b, widened, perm, off, 0.01)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(a, mixing.step_dense(X, widened, perm, off, 0.01).astype(np.float32))


# ---------------------------------------------------------------- consensus

def test_consensus_against_numpy_and_frobenius_identity():
    W, P = 8, 1000
    X = rng_stack(17, W, P + 5)
    d = oracle.consensus(X, P)
    Xd = X[:, :P].astype(np.float64)
    want = np.linalg.norm(Xd - Xd.mean(0), axis=1)
    np.testing.assert_allclose(d, want, rtol=1e-13)
    # sum_i d_i^2 = ||X||_F^2 - W ||xbar||^2
    np.testing.assert_allclose((d**2).sum(), (Xd**2).sum() - W * (Xd.mean(0)**2).sum(), rtol=1e-12)


def test_consensus_is_zero_for_identical_models():
    for W in (3, 8, 13):
        X = np.tile(rng_stack(18, 1, 257), (W, 1))
        np.testing.assert_array_equal(oracle.consensus(X), np.zeros(W))


def test_consensus_single_outlier_closed_form():
    # all rows equal to a except row j = a + e: d_j = (W-1)/W ||e||, others ||e||/W
    W, P, j = 5, 64, 2
    a = rng_stack(19, 1, P)[0]
    e = np.zeros(P, dtype=np.float32)
    e[:8] = 0.5                       # exactly representable sums
    X = np.tile(a, (W, 1))
    X[j] = a + e
    e_eff = (X[j] - a).astype(np.float64)
    d = oracle.consensus(X)
    n = np.linalg.norm(e_eff)
    want = np.full(W, n / W)
    want[j] = n * (W - 1) / W
    np.testing.assert_allclose(d, want, rtol=1e-6)


def test_consensus_expectation_after_first_step():
    # identical init, g_i = mu + 0.5 z_i: x_i - xbar = -lr*0.5*(zbar_group - zbar_all),
    # so E d_i^2 = P lr^2 0.25 (1/|g| - 1/W)
    W, P, lr, gsz = 8, 200000, 0.01, 4
    r = np.random.default_rng(21)
    x0 = (0.02 * r.standard_normal(P)).astype(np.float32)
    mu = r.standard_normal(P)
    G = (mu + 0.5 * r.standard_normal((W, P))).astype(np.float32)
    X = np.tile(x0, (W, 1))
    perm, off = oracle.partition(0, 0, W, [gsz, gsz])
    oracle.step(X, G, perm, off, lr)
    d = oracle.consensus(X)
    want = np.sqrt(P * lr**2 * 0.25 * (1.0 / gsz - 1.0 / W))
    np.testing.assert_allclose(d, want, rtol=0.02)


def test_lemma1_bound_on_the_rack_pattern():
    # pure averaging with the periodic rack pattern (period B = 4): after k periods
    # every worker is within rho^k ||X_0||^2 of the true average (squared norms)
    W, P, B = 8, 48, 4
    X0 = rng_stack(22, W, P)
    mats = [mixing.mixing_matrix(*rack_pattern(k)) for k in range(B)]
    M = mixing.product(mats)
    rho = mixing.second_eigenvalue(M)
    sigma = mixing.contraction_norm(M)
    assert 0.0 < rho < 1.0 and rho <= sigma + 1e-12 and sigma < 1.0
    X = X0.copy()
    Z = np.zeros_like(X)
    fro2 = float((X0.astype(np.float64)**2).sum())
    prev = oracle.consensus(X)
    for k in range(1, 7):
        for b in range(B):
            perm, off = rack_pattern(b)
            oracle.step(X, Z, perm, off, 0.0)
        d = oracle.consensus(X)
        slack = 1e-9
        assert np.all(d**2 <= sigma**(2 * k) * fro2 + slack)      # rigorous form
        assert np.all(d**2 <= rho**k * fro2 + slack)              # as Lemma 1 states it
        assert d.max() <= prev.max() + 1e-7                       # and it contracts
        prev = d
    assert prev.max() < 1e-2 * oracle.consensus(X0).max()


def test_scaled_error_yardstick_against_its_definition():
    # the parity yardstick is |a-b| / max(|b|, rms(b row)): numpy statement, hand values, window, NaN
    r = np.random.default_rng(9)
    want = r.normal(0, 0.02, (5, 1000)).astype(np.float32)
    got = (want.astype(np.float64) * (1 + r.normal(0, 1e-6, want.shape))).astype(np.float32)
    w64, g64 = want.astype(np.float64), got.astype(np.float64)
    den = np.maximum(np.abs(w64), np.sqrt((w64**2).mean(axis=1, keepdims=True)))
    np.testing.assert_allclose(oracle.scaled_error(got, want), (np.abs(g64 - w64) / den).max(), rtol=1e-12)
    assert oracle.scaled_error(want, want) == 0.0
    # one element off by 3 in a row of rms sqrt((3*1 + 25)/4): the rms is the denominator for a small element ...
    b = np.array([[1, 1, 1, 5]], dtype=np.float32)
    a = b.copy()
    a[0, 0] += 3
    assert abs(oracle.scaled_error(a, b) - 3 / np.sqrt(7.0)) < 1e-12
    # ... and the element itself for a large one
    a = b.copy()
    a[0, 3] += 1
    assert abs(oracle.scaled_error(a, b) - 1 / 5) < 1e-12
    # a window looks at its own columns only, for the error and for the rms
    a = b.copy()
    a[0, 3] += 1
    assert oracle.scaled_error(a, b, 0, 3) == 0.0
    assert abs(oracle.scaled_error(a, b, 2, 2) - 1 / 5) < 1e-12
    a[0, 1] = np.nan
    assert np.isnan(oracle.scaled_error(a, b))
