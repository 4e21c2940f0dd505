"""Pins for the oracle's master update (CPU only).

What fixes it: the definition of the proximal operator (Section 2, notation), the
update of Alg. 1 (master (ii)), the momentum update of Alg. 3 and the two identities
used in its analysis: x_{t+1} - x_t = theta (y_{t+1} - y_t) and
x_{t+1} = theta y_{t+1} + (1 - theta) snapshot.
"""
import numpy as np
import pytest

import oracle


def _setup(M=5, d=300, b=8, seed=0):
    rng = np.random.default_rng(seed)
    codes = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d)).astype(np.int8)
    delta = (rng.random(M) * 1e-2).astype(np.float32)
    g = rng.standard_normal(d).astype(np.float32)
    x = rng.standard_normal(d).astype(np.float32)
    return codes, delta, g, x, rng


def test_prox_is_the_argmin():
    # prox_{eta h}(z) = argmin_y h(y) + |y - z|^2/(2 eta), h = l1*|y|, by brute force on a grid
    eta, l1 = np.float32(0.5), np.float32(0.3)
    zs = np.array([-2.0, -0.2, -0.15, 0.0, 0.1, 0.15, 0.151, 1.0, 3.0], dtype=np.float32)
    grid = np.linspace(-4, 4, 800001)
    for z in zs:
        # one worker, code 0: u = g, and x - eta*g = z with g = 0
        x = np.array([z], dtype=np.float32)
        oracle.master_update(np.zeros((1, 1), dtype=np.int8), np.ones(1, dtype=np.float32), 1.0,
                             np.zeros(1, dtype=np.float32), x, eta=eta, l1=l1)
        obj = float(l1) * np.abs(grid) + (grid - float(z)) ** 2 / (2 * float(eta))
        assert abs(x[0] - grid[np.argmin(obj)]) < 2e-5
    # l1 = 0: identity
    x = zs.copy()
    oracle.master_update(np.zeros((1, zs.size), dtype=np.int8), np.ones(1, dtype=np.float32), 1.0,
                         np.zeros(zs.size, dtype=np.float32), x, eta=eta, l1=0.0)
    assert np.array_equal(x, zs)


def test_update_against_float64_formula():
    codes, delta, g, x, _ = _setup()
    M, d = codes.shape
    eta, l1 = 0.05, 0.01
    x0 = x.copy()
    oracle.master_update(codes, delta, np.float32(1.0 / M), g, x, eta=eta, l1=l1)
    gbar = (delta.astype(np.float64)[:, None] * codes.astype(np.float64)).sum(0) / M
    z = x0 - float(np.float32(eta)) * (gbar + g)
    kappa = float(np.float32(eta)) * float(np.float32(l1))
    want = np.sign(z) * np.maximum(np.abs(z) - kappa, 0)
    assert np.allclose(x, want, rtol=0, atol=3e-7 * np.abs(x0).max())
    # gradient mapping G_eta(x) = (x - prox(x - eta*u))/eta equals u when h = 0
    x = x0.copy()
    oracle.master_update(codes, delta, np.float32(1.0 / M), g, x, eta=eta, l1=0.0)
    assert np.allclose((x0 - x) / float(np.float32(eta)), gbar + g, rtol=0, atol=2e-5)


def test_single_worker_reduces_to_prox_svrg_step():
    codes, delta, g, x, _ = _setup(M=1)
    x0 = x.copy()
    oracle.master_update(codes, delta, 1.0, g, x, eta=0.1, l1=0.0)
    u = oracle.dequantize(codes[0], delta[0]) + g               # Q(alpha) + grad f(snapshot)
    want = x0 - np.float32(0.1) * u
    assert np.array_equal(x, want)


def test_sum_versus_mean_scale():
    codes, delta, g, x, _ = _setup(M=4)
    xa, xb = x.copy(), x.copy()
    oracle.master_update(codes, delta, 0.25, g, xa, eta=0.1)
    oracle.master_update(codes, (delta * np.float32(0.25)), 1.0, g, xb, eta=0.1)   # 1/4 is exact
    assert np.array_equal(xa, xb)


def test_momentum_update_and_identities():
    codes, delta, g, x, rng = _setup(M=3, d=500)
    d = x.size
    xs = rng.standard_normal(d).astype(np.float32)
    y = rng.standard_normal(d).astype(np.float32)
    theta, eta, l1 = np.float32(0.5), np.float32(0.2), np.float32(0.01)
    x = oracle.acc_mix(y, xs, theta)
    xsum = np.zeros(d, dtype=np.float32)
    x_prev, y_prev = x.copy(), y.copy()
    oracle.master_update(codes, delta, np.float32(1 / 3), g, x, y, xs, xsum, eta=eta, theta=theta, l1=l1)
    # y follows the plain proximal step
    y_ref = y_prev.copy()
    oracle.master_update(codes, delta, np.float32(1 / 3), g, y_ref, eta=eta, l1=l1)
    assert np.array_equal(y, y_ref)
    tol = 4e-7 * max(np.abs(y).max(), np.abs(xs).max())
    assert np.allclose(x, theta * y.astype(np.float64) + (1 - theta) * xs.astype(np.float64), rtol=0, atol=tol)
    assert np.allclose(x.astype(np.float64) - x_prev, theta * (y.astype(np.float64) - y_prev), rtol=0, atol=tol)
    assert np.array_equal(xsum, x)
    oracle.master_update(codes, delta, np.float32(1 / 3), g, x, y, xs, xsum, eta=eta, theta=theta, l1=l1)
    assert np.allclose(oracle.acc_snapshot(xsum, 2), (x_prev * 0 + (xsum.astype(np.float64)) / 2), atol=1e-7)
    # y equal to the snapshot: the mix returns the snapshot bit for bit (flag-bit case of Section 4.1)
    assert np.array_equal(oracle.acc_mix(xs, xs, np.float32(2 / 3)).view(np.uint32), xs.view(np.uint32))


def test_mu_terms():
    rng = np.random.default_rng(8)
    x = rng.standard_normal(100).astype(np.float32)
    xs = rng.standard_normal(100).astype(np.float32)
    k, dlt, _ = oracle.quantize(x, 8, 1, 2, oracle.MASTER_ID, oracle.TAG_MODEL)
    e, r = oracle.mu_terms(k, dlt, x, xs)
    q = oracle.dequantize(k, dlt).astype(np.float64)
    assert np.isclose(e, np.sum((q - x) ** 2)) and np.isclose(r, np.sum((x.astype(np.float64) - xs) ** 2))
    assert e <= 100 * float(dlt) ** 2              # each coordinate moves by less than delta
