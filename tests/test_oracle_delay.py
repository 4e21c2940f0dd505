"""Pins for the oracle's bounded-delay emulation (CPU only): Assumption 3 / Section 3.2 of the paper."""
import numpy as np

import oracle
from oracle import algorithms as alg
import synth


def test_worker_delay_groups():
    assert [alg.worker_delay(w, 8, 0) for w in range(8)] == [0] * 8
    assert [alg.worker_delay(w, 8, 1) for w in range(8)] == [0, 0, 0, 0, 1, 1, 1, 1]
    assert [alg.worker_delay(w, 8, 3) for w in range(8)] == [0, 0, 1, 1, 2, 2, 3, 3]
    assert [alg.worker_delay(w, 4, 3) for w in range(4)] == [0, 1, 2, 3]
    assert max(alg.worker_delay(w, 5, 2) for w in range(5)) == 2          # never more than tau


def test_zero_delay_is_the_synchronous_loop():
    p = synth.dense_logistic(120, 16, seed=1)
    a = alg.run(p, "asylpg", 4, 4, 8, 8, 6, 2, 0.3, seed=3)
    b = alg.run(p, "asylpg", 4, 4, 8, 8, 6, 2, 0.3, seed=3, tau=0)
    assert np.array_equal(a.x, b.x)


def test_delayed_run_against_float64_delayed_prox_svrg():
    """Unquantized (b = b_x = 32) so that only the delay structure is under test."""
    p = synth.dense_logistic(300, 24, seed=2, l2=1e-3, l1=1e-4)
    M, B, m, S, lr, tau = 4, 6, 12, 2, 0.4, 3
    tr = alg.run(p, "asylpg", M, B, 32, 32, m, S, lr, seed=7, tau=tau)
    X, y = p.dense.astype(np.float64), p.y.astype(np.float64)
    l2, l1 = float(np.float32(p.l2)), float(np.float32(p.l1))
    slope = lambda z, t: -t / (1 + np.exp(t * z))
    xs = np.zeros(p.d)
    for e in range(S):
        x = xs.copy()
        g = X.T @ slope(X @ xs, y) / p.n + l2 * xs
        hist = []
        for t in range(m):
            hist.append(x.copy())
            u = g.copy()
            for w in range(M):
                xd = hist[max(0, t - (w * (tau + 1)) // M)]                 # the model worker w saw
                idx = oracle.sample_indices(p.n, B, 7, e * m + t, w)
                A = X[idx]
                u += (A.T @ (slope(A @ xd, y[idx]) - slope(A @ xs, y[idx])) / B + l2 * (xd - xs)) / M
            z = x - lr * u
            x = np.sign(z) * np.maximum(np.abs(z) - lr * l1, 0)
        xs = x
    assert np.linalg.norm(tr.x_snap - xs) < 1e-5 * np.linalg.norm(xs)
    # the delay changes the trajectory (otherwise this test would not see it)
    sync = alg.run(p, "asylpg", M, B, 32, 32, m, S, lr, seed=7)
    assert np.linalg.norm(sync.x_snap - tr.x_snap) > 1e-4 * np.linalg.norm(xs)
    assert tr.objectives[-1] < tr.objectives[0]


def test_stale_workers_see_the_snapshot_at_the_epoch_start():
    # tau + 1 = M: worker w is w rounds behind; in round t < w it still holds the snapshot (flag bit): alpha = 0
    p = synth.dense_logistic(100, 10, seed=3)
    M, tau = 3, 2
    full = alg.run(p, "asylpg", M, 4, 32, 32, m=2, S=1, lr=0.5, seed=1, tau=tau)
    rp = oracle.RefProblem(p)
    x0 = np.zeros(p.d, dtype=np.float32)
    g = oracle.full_grad(rp, x0)
    x1 = x0 - np.float32(0.5) * g                                   # round 0: every worker sends 0
    # round 1: worker 0 uses x1, worker 1 uses x0 (snapshot, alpha = 0), worker 2 uses x0
    a0 = oracle.vr_grad(rp, oracle.sample_indices(p.n, 4, 1, 1, 0), x1, x0)
    grads = np.stack([a0, np.zeros_like(a0), np.zeros_like(a0)])
    x2 = x1.copy()
    oracle.master_update_full(grads, np.float32(1 / 3), g, x2, eta=0.5)
    assert np.array_equal(full.x, x2)
