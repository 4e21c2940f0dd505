"""Pins for the oracle's "one master update per received gradient" mode (CPU only).

Alg. 1 states the master's rule for a single received gradient; a round of M workers applied that way is
M such updates in worker order.  What fixes it: it is the already pinned single-message update composed M
times; closed forms without a prox; a float64 loop; M = 1 coincides with the mean mode.
"""
import numpy as np
import pytest

import oracle
from oracle import algorithms as alg
import synth


def _inputs(M, d, seed):
    rng = np.random.default_rng(seed)
    k = rng.integers(-128, 128, size=(M, d)).astype(np.int8)
    delta = (rng.random(M) * 1e-2).astype(np.float32)
    g = (0.1 * rng.standard_normal(d)).astype(np.float32)
    x, xs, y, sm = (rng.standard_normal(d).astype(np.float32) for _ in range(4))
    return k, delta, g, x, xs, y, sm


@pytest.mark.parametrize("acc", [False, True])
def test_each_is_the_single_message_update_composed(acc):
    M, d = 5, 37
    k, delta, g, x0, xs, y0, s0 = _inputs(M, d, 1)
    eta, theta, l1 = np.float32(0.3), np.float32(0.4), np.float32(0.05)
    x, y, sm = x0.copy(), y0.copy(), s0.copy()
    if acc:
        oracle.master_update_each(k, delta, g, x, y, xs, sm, eta=eta, theta=theta, l1=l1)
    else:
        oracle.master_update_each(k, delta, g, x, eta=eta, l1=l1)
    xr, yr, sr = x0.copy(), y0.copy(), s0.copy()
    for w in range(M):                              # the pinned update, one message (M = 1, scale 1) at a time
        if acc:
            oracle.master_update(k[w:w + 1], delta[w:w + 1], np.float32(1), g, xr, yr, xs, sr, eta=eta, theta=theta, l1=l1)
        else:
            oracle.master_update(k[w:w + 1], delta[w:w + 1], np.float32(1), g, xr, eta=eta, l1=l1)
    assert np.array_equal(x, xr)
    if acc:
        assert np.array_equal(y, yr) and np.array_equal(sm, sr)
        # Alg. 3: x = theta y + (1 - theta) snapshot after the last update
        assert np.allclose(x, theta * y + (1 - theta) * xs, rtol=0, atol=1e-6)


def test_each_with_one_worker_is_the_mean_mode():
    k, delta, g, x0, xs, y0, s0 = _inputs(1, 50, 2)
    a, b = x0.copy(), x0.copy()
    oracle.master_update_each(k, delta, g, a, eta=0.2, l1=0.01)
    oracle.master_update(k, delta, np.float32(1), g, b, eta=0.2, l1=0.01)
    assert np.array_equal(a, b)


def test_each_without_prox_is_a_sum_of_steps():
    # h = 0: x_M = x_0 - eta * sum_w (delta_w k_w + g)  exactly in real arithmetic
    M, d = 7, 64
    k, delta, g, x0, *_ = _inputs(M, d, 3)
    x = x0.copy()
    oracle.master_update_each(k, delta, g, x, eta=0.05, l1=0.0)
    eta = float(np.float32(0.05))
    want = x0.astype(np.float64) - eta * ((delta.astype(np.float64)[:, None] * k).sum(0) + M * g.astype(np.float64))
    assert np.max(np.abs(x - want)) < 1e-6 * np.max(np.abs(want))
    # and it differs from one step with the mean by the factor M in the step size
    xm = x0.copy()
    oracle.master_update(k, delta, np.float32(1.0), g, xm, eta=0.05, l1=0.0)      # one step with the sum, g added once
    assert np.max(np.abs(xm - x)) > 1e-3


def test_each_full_precision_messages_match_codes_on_exact_inputs():
    # gradients that are exactly delta*k: the float path must give the same bits as the code path
    M, d = 4, 33
    k, _, g, x0, xs, y0, s0 = _inputs(M, d, 4)
    delta = np.array([2.0 ** -7, 2.0 ** -5, 2.0 ** -9, 2.0 ** -6], dtype=np.float32)
    grads = (delta[:, None] * k).astype(np.float32)
    a, ya, sa = x0.copy(), y0.copy(), s0.copy()
    b, yb, sb = x0.copy(), y0.copy(), s0.copy()
    oracle.master_update_each(k, delta, g, a, ya, xs, sa, eta=0.3, theta=0.5, l1=0.02)
    oracle.master_update_each_full(grads, g, b, yb, xs, sb, eta=0.3, theta=0.5, l1=0.02)
    assert np.array_equal(a, b) and np.array_equal(ya, yb) and np.array_equal(sa, sb)


def test_loop_with_one_update_per_gradient_against_float64():
    """Unquantized so that only the order of the updates is under test."""
    p = synth.dense_logistic(300, 24, seed=5, l2=1e-3, l1=1e-4)
    M, B, m, S, lr = 4, 6, 10, 2, 0.1
    tr = alg.run(p, "asylpg", M, B, 32, 32, m, S, lr, seed=9, each=True)
    X, y = p.dense.astype(np.float64), p.y.astype(np.float64)
    l2, l1 = float(np.float32(p.l2)), float(np.float32(p.l1))
    lr64 = float(np.float32(lr))
    slope = lambda z, t: -t / (1 + np.exp(t * z))
    xs = np.zeros(p.d)
    for e in range(S):
        x = xs.copy()
        g = X.T @ slope(X @ xs, y) / p.n + l2 * xs
        for t in range(m):
            xr = x.copy()                                   # the model all M workers read this round
            for w in range(M):
                idx = oracle.sample_indices(p.n, B, 9, e * m + t, w)
                A = X[idx]
                u = g + A.T @ (slope(A @ xr, y[idx]) - slope(A @ xs, y[idx])) / B + l2 * (xr - xs)
                z = x - lr64 * u
                x = np.sign(z) * np.maximum(np.abs(z) - lr64 * l1, 0)
        xs = x
    assert np.linalg.norm(tr.x_snap - xs) < 1e-5 * np.linalg.norm(xs)
    mean_mode = alg.run(p, "asylpg", M, B, 32, 32, m, S, lr, seed=9)
    assert np.linalg.norm(mean_mode.x_snap - tr.x_snap) > 1e-3 * np.linalg.norm(xs)
    assert tr.objectives[-1] < tr.objectives[0]


def test_loop_one_worker_is_unchanged_and_acc_snapshot_averages_all_iterates():
    p = synth.dense_logistic(120, 16, seed=1)
    a = alg.run(p, "asylpg", 1, 4, 8, 8, 6, 2, 0.3, seed=3)
    b = alg.run(p, "asylpg", 1, 4, 8, 8, 6, 2, 0.3, seed=3, each=True)
    assert np.array_equal(a.x, b.x) and a.bits_up == b.bits_up
    # Alg. 3 with M updates per round: the snapshot stays inside the hull of the iterates (a mean, not a sum)
    c = alg.run(p, "acc", 3, 4, 8, 8, 5, 2, 0.1, seed=3, each=True)
    assert np.isfinite(c.objectives[-1]) and c.objectives[-1] < c.objectives[0]
    assert np.abs(c.x_snap).max() < 10 * max(1e-3, np.abs(c.x).max())
