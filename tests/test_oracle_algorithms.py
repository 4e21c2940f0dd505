"""Pins for the oracle's epoch loops, Algorithms 1-3 (CPU only).

The paper prints no trajectory values, so the loops are pinned by structure: message
sizes (Section 3.1: 32 + b*d bits; Section 4.2: 32 + nnz*(log d + b) bits), the flag-bit
case of Section 4.1, descent of the objective, and closeness of the low-precision run
to a full-precision proximal-SVRG written here in numpy on the same sampled indices
(Section 5.1 reports similar convergence).  Trajectory values themselves are
otherwise unpinned.
"""
import math

import numpy as np
import pytest

import oracle
from oracle import algorithms as alg
import synth


def _full_precision_svrg(p, M, B, m, S, lr, seed):
    """Mini-batch proximal SVRG in float64 with the oracle's index streams, no quantization."""
    X = p.dense.astype(np.float64)
    y = p.y.astype(np.float64)
    l2, l1 = float(np.float32(p.l2)), float(np.float32(p.l1))

    def slope(z, yy):
        return -yy / (1 + np.exp(yy * z))

    xs = np.zeros(p.d)
    for e in range(S):
        x = xs.copy()
        g = X.T @ slope(X @ xs, y) / p.n + l2 * xs
        for t in range(m):
            it = e * m + t
            u = np.zeros(p.d)
            for w in range(M):
                idx = oracle.sample_indices(p.n, B, seed, it, w)
                A = X[idx]
                r = slope(A @ x, y[idx]) - slope(A @ xs, y[idx])
                u += (A.T @ r / B + l2 * (x - xs)) / M
            z = x - lr * (u + g)
            x = np.sign(z) * np.maximum(np.abs(z) - lr * l1, 0)
        xs = x
    return xs


def _obj64(p, x):
    m = p.y.astype(np.float64) * (p.dense.astype(np.float64) @ x)
    return np.mean(np.logaddexp(0, -m)) + 0.5 * float(np.float32(p.l2)) * x @ x \
        + float(np.float32(p.l1)) * np.abs(x).sum()


def test_asylpg_tracks_full_precision_and_counts_bits():
    p = synth.dense_logistic(300, 40, seed=1, l2=1e-3, l1=1e-4)
    M, B, m, S, lr, bx, b = 3, 8, 30, 2, 0.5, 8, 8
    tr = alg.run(p, "asylpg", M, B, bx, b, m, S, lr, seed=5)
    assert len(tr.objectives) == S + 1
    assert abs(tr.objectives[0] - math.log(2)) < 1e-12
    assert tr.objectives[2] < tr.objectives[1] < tr.objectives[0]
    ref = _full_precision_svrg(p, M, B, m, S, lr, seed=5)
    assert abs(tr.objectives[-1] - _obj64(p, ref)) < 0.02 * _obj64(p, ref)
    assert np.linalg.norm(tr.x_snap - ref) < 0.1 * np.linalg.norm(ref)
    # message sizes; the first round of each epoch is the flag-bit case
    assert tr.bits_up == S * m * M * (32 + b * p.d)
    assert tr.bits_down == S * (1 + (m - 1) * (32 + bx * p.d))


def test_first_round_of_an_epoch_uses_the_snapshot_gradient():
    # with m = 1 every round is the flag-bit round: alpha = 0, u = grad f(snapshot): plain proximal gradient
    p = synth.dense_logistic(100, 12, seed=2, l2=1e-2, l1=0.0)
    tr = alg.run(p, "asylpg", 2, 4, 8, 8, m=1, S=3, lr=0.5, seed=0)
    rp = oracle.RefProblem(p)
    x = np.zeros(p.d, dtype=np.float32)
    for _ in range(3):
        x = x - np.float32(0.5) * oracle.full_grad(rp, x)
    assert np.array_equal(tr.x_snap, x)
    assert tr.bits_down == 3


def test_sparse_variant_sends_fewer_bits_and_converges():
    p = synth.sparse_text_logistic(400, 300, mean_nnz=8, seed=3, l2=1e-3, l1=1e-5)
    M, B, m, S, lr = 2, 8, 25, 2, 1.0
    dense_run = alg.run(p, "asylpg", M, B, 8, 4, m, S, lr, seed=1)
    sparse_run = alg.run(p, "sparse", M, B, 8, 4, m, S, lr, seed=1)
    assert sparse_run.bits_up < dense_run.bits_up
    assert sparse_run.objectives[-1] < sparse_run.objectives[0]
    assert dense_run.objectives[-1] < dense_run.objectives[0]
    per_msg = 32 + 4 * p.d
    assert dense_run.bits_up == S * m * M * per_msg


def test_accelerated_variant():
    p = synth.dense_logistic(300, 30, seed=4, l2=1e-3, l1=0.0)
    M, B, m, S, lr = 2, 8, 20, 3, 0.2
    tr = alg.run(p, "acc", M, B, 8, 8, m, S, lr, seed=2)
    assert tr.objectives[-1] < tr.objectives[1] < tr.objectives[0]
    # first epoch starts at the snapshot (y_0 = snapshot): one flag bit; later epochs start elsewhere
    assert tr.bits_down == 1 + (S * m - 1) * (32 + 8 * p.d)
    # full-precision Alg. 3 in float64 on the same index streams
    X, yy, l2 = p.dense.astype(np.float64), p.y.astype(np.float64), float(np.float32(p.l2))
    slope = lambda z, t: -t / (1 + np.exp(t * z))
    xs = np.zeros(p.d)
    y = xs.copy()
    for s in range(1, S + 1):
        theta = 2.0 / (s + 2)
        eta = lr / theta
        x = theta * y + (1 - theta) * xs
        g = X.T @ slope(X @ xs, yy) / p.n + l2 * xs
        xsum = np.zeros(p.d)
        for t in range(m):
            u = g.copy()
            for w in range(M):
                idx = oracle.sample_indices(p.n, B, 2, (s - 1) * m + t, w)
                A = X[idx]
                u += (A.T @ (slope(A @ x, yy[idx]) - slope(A @ xs, yy[idx])) / B + l2 * (x - xs)) / M
            y = y - eta * u
            x = xs + theta * (y - xs)
            xsum += x
        xs = xsum / m
    assert np.linalg.norm(tr.x_snap - xs) < 0.1 * np.linalg.norm(xs)
    assert abs(tr.objectives[-1] - _obj64(p, xs)) < 0.02 * _obj64(p, xs)


def test_reproducible():
    p = synth.dense_logistic(80, 10, seed=5)
    a = alg.run(p, "sparse", 2, 4, 8, 4, 5, 2, 0.3, seed=9)
    b = alg.run(p, "sparse", 2, 4, 8, 4, 5, 2, 0.3, seed=9)
    c = alg.run(p, "sparse", 2, 4, 8, 4, 5, 2, 0.3, seed=10)
    assert np.array_equal(a.x, b.x) and a.bits_up == b.bits_up
    assert not np.array_equal(a.x, c.x)
