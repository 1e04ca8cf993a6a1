"""Pins for the oracle's step with momentum / weight decay and the SWA
ensemble (CPU only): reduction to the plain step, torch.optim.SGD as the
library statement of the local optimizer, closed forms, locality of the
momentum buffer, and the exponential moving average of Listing 1 with its
final average over all workers."""
import numpy as np
import pytest
import torch

import oracle
from oracle import mixing


def stacks(seed, W, P):
    r = np.random.default_rng(seed)
    return ((0.02 * r.standard_normal((W, P))).astype(np.float32), r.standard_normal((W, P)).astype(np.float32))


def test_reduces_to_the_plain_step():
    W, P = 8, 33
    X, G = stacks(1, W, P)
    perm, off = oracle.partition(3, 0, W, [2, 3, 3])
    a, b = X.copy(), X.copy()
    V = np.zeros_like(X)
    oracle.step(a, G, perm, off, 0.01)
    oracle.step_opt(b, G, perm, off, 0.01, V=V, momentum=0.0, weight_decay=0.0)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(V, G)             # the buffer then just holds the gradient
    c = X.copy()
    oracle.step_opt(c, G, perm, off, 0.01)          # no buffers at all
    np.testing.assert_array_equal(a, c)


@pytest.mark.parametrize("momentum,weight_decay", [(0.9, 0.0), (0.9, 5e-4), (0.0, 1e-2), (0.5, 0.1)])
def test_local_optimizer_matches_torch_sgd(momentum, weight_decay):
    # W independent torch optimizers (fp64), then the group mean with numpy
    W, P, T, lr = 6, 17, 4, 0.05
    X, _ = stacks(2, W, P)
    V = np.zeros_like(X)
    params = [torch.nn.Parameter(torch.tensor(X[i], dtype=torch.float64)) for i in range(W)]
    opts = [torch.optim.SGD([p], lr=float(np.float32(lr)), momentum=float(np.float32(momentum)),
                            weight_decay=float(np.float32(weight_decay))) for p in params]
    for t in range(T):
        _, G = stacks(10 + t, W, P)
        perm, off = oracle.partition(5, t, W, [3, 3])
        oracle.step_opt(X, G, perm, off, lr, V=V, momentum=momentum, weight_decay=weight_decay)
        for i in range(W):
            params[i].grad = torch.tensor(G[i], dtype=torch.float64)
            opts[i].step()
        with torch.no_grad():
            for members in mixing.groups_of(perm, off):
                m = torch.stack([params[i].data for i in members]).mean(0)
                for i in members:
                    params[i].data.copy_(m.to(torch.float32).to(torch.float64))   # replicas are stored as fp32
        want = np.stack([p.detach().numpy() for p in params])
        np.testing.assert_allclose(X, want, rtol=0, atol=2e-7 * (t + 1))
        if momentum:
            bufs = np.stack([opts[i].state[params[i]]["momentum_buffer"].numpy() for i in range(W)])
            np.testing.assert_allclose(V, bufs, rtol=2e-6, atol=1e-6)


def test_constant_gradient_closed_form():
    # groups of one, no decay: v_t = g (1 - mu^t)/(1 - mu), x_t = x_0 - lr * sum_s v_s
    W, P, T, lr, mu = 3, 9, 6, 0.1, 0.8
    X, G = stacks(4, W, P)
    x0 = X.astype(np.float64)
    V = np.zeros_like(X)
    perm, off = oracle.partition(0, 0, W, [1] * W)
    mu32, lr32 = float(np.float32(mu)), float(np.float32(lr))
    drift = np.zeros_like(x0)
    for t in range(1, T + 1):
        oracle.step_opt(X, G, perm, off, lr, V=V, momentum=mu)
        v_t = G.astype(np.float64) * (1 - mu32**t) / (1 - mu32)
        np.testing.assert_allclose(V, v_t, rtol=1e-6)
        drift += v_t
        np.testing.assert_allclose(X, x0 - lr32 * drift, rtol=0, atol=1e-6)


def test_momentum_buffer_is_local_to_the_worker():
    W, P = 4, 12
    X, G = stacks(5, W, P)
    perm, off = oracle.partition(1, 0, W, [4])
    V1 = np.full_like(X, 0.5)
    V2 = V1.copy()
    G2 = G.copy()
    G2[2] += 7.0                                   # another worker of the same group gets a different gradient
    a, b = X.copy(), X.copy()
    oracle.step_opt(a, G, perm, off, 0.01, V=V1, momentum=0.9)
    oracle.step_opt(b, G2, perm, off, 0.01, V=V2, momentum=0.9)
    for i in (0, 1, 3):
        np.testing.assert_array_equal(V1[i], V2[i])     # buffers are never averaged
    assert not np.array_equal(V1[2], V2[2])
    assert not np.array_equal(a, b)                      # while the parameters are


def test_swa_is_the_moving_average_of_the_synchronised_models():
    W, P, T, f = 8, 21, 5, 0.75
    X, _ = stacks(6, W, P)
    S = X.copy()
    s0 = S.astype(np.float64)
    f32 = float(np.float32(f))
    history = []
    for t in range(T):
        _, G = stacks(20 + t, W, P)
        perm, off = oracle.partition(2, t, W, [4, 4])
        oracle.step_opt(X, G, perm, off, 0.01, S=S, factor=f)
        history.append(X.astype(np.float64).copy())
    want = f32**T * s0
    for t, Xt in enumerate(history):
        want += (1 - f32) * f32**(T - 1 - t) * Xt
    np.testing.assert_allclose(S, want, rtol=0, atol=1e-6)
    # the final model of Listing 1: the SWA models averaged over all workers (one group of W, no update)
    perm, off = oracle.partition(0, 0, W, [W])
    final = S.copy()
    oracle.step(final, np.zeros_like(S), perm, off, 0.0)
    np.testing.assert_allclose(final[0], S.astype(np.float64).mean(0), rtol=0, atol=1e-7)
    assert all(np.array_equal(final[0], final[i]) for i in range(W))


def test_swa_factor_extremes_and_fixed_point():
    W, P = 4, 10
    X, G = stacks(7, W, P)
    perm, off = oracle.partition(0, 1, W, [2, 2])
    S = np.full_like(X, 3.0)
    a = X.copy()
    oracle.step_opt(a, G, perm, off, 0.01, S=S, factor=0.0)
    np.testing.assert_array_equal(S, a)                  # factor 0: the SWA model is the new model
    S1 = np.full_like(X, 3.0)
    b = X.copy()
    oracle.step_opt(b, G, perm, off, 0.01, S=S1, factor=1.0)
    np.testing.assert_array_equal(S1, np.full_like(X, 3.0))   # factor 1: it never moves
    np.testing.assert_array_equal(a, b)                  # and it never feeds back into the model
