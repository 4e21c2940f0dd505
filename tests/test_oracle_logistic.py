"""Pins for the oracle's objective, full gradient and variance-reduced gradient (CPU only).

What fixes them: problem (1) of the paper with the logistic loss of Section 5.1,
finite differences, closed forms at x = 0, dense/CSR equivalence, and the structure
of the SVRG-style difference in Alg. 1 (worker (i)) together with Assumption 1.
"""
import numpy as np
import pytest

import oracle
import synth


def _small_dense(n=40, d=7, seed=0, l2=1e-2):
    return synth.dense_logistic(n, d, seed=seed, l2=l2, l1=0.0)


def _small_csr(n=60, d=50, seed=0, l2=1e-2):
    return synth.sparse_text_logistic(n, d, mean_nnz=6.0, seed=seed, l2=l2, l1=0.0)


def _densify(p):
    X = np.zeros((p.n, p.d), dtype=np.float32)
    for i in range(p.n):
        s, e = p.indptr[i], p.indptr[i + 1]
        X[i, p.indices[s:e]] = p.values[s:e]
    return synth.Problem(n=p.n, d=p.d, y=p.y, l2=p.l2, l1=p.l1, dense=X)


def _numpy_objective(X, y, x, l2, l1):
    m = y.astype(np.float64) * (X.astype(np.float64) @ x.astype(np.float64))
    return np.mean(np.logaddexp(0.0, -m)) + 0.5 * l2 * np.sum(x.astype(np.float64) ** 2) \
        + l1 * np.sum(np.abs(x.astype(np.float64)))


def _numpy_grad(X, y, x, l2):
    X64, y64, x64 = X.astype(np.float64), y.astype(np.float64), x.astype(np.float64)
    m = y64 * (X64 @ x64)
    s = -y64 / (1.0 + np.exp(m))
    return X64.T @ s / X.shape[0] + l2 * x64


def test_closed_forms_at_zero():
    p = _small_dense()
    rp = oracle.RefProblem(p)
    x0 = np.zeros(p.d, dtype=np.float32)
    assert abs(oracle.objective(rp, x0) - np.log(2.0)) < 1e-12
    g = oracle.full_grad(rp, x0)
    want = -(p.dense.astype(np.float64).T @ p.y.astype(np.float64)) / (2 * p.n)   # slope at margin 0 is -y/2
    assert np.allclose(g, want, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("make", [_small_dense, _small_csr])
def test_full_grad_matches_finite_differences(make):
    p = make()
    rp = oracle.RefProblem(p)
    rng = np.random.default_rng(1)
    x = (0.5 * rng.standard_normal(p.d)).astype(np.float32)
    g = oracle.full_grad(rp, x)
    h = 2.0 ** -8                                  # exactly representable steps
    for j in rng.choice(p.d, size=min(p.d, 7), replace=False):
        xp, xm = x.copy(), x.copy()
        xp[j] += np.float32(h)
        xm[j] -= np.float32(h)
        step = float(xp[j]) - float(xm[j])
        fd = (oracle.objective(rp, xp) - oracle.objective(rp, xm)) / step
        assert abs(fd - g[j]) < 2e-5 * max(1.0, abs(fd)), (j, fd, g[j])


def test_objective_and_grad_against_numpy_dense_and_l1():
    p = synth.dense_logistic(50, 9, seed=3, l2=3e-2, l1=2e-2)
    rp = oracle.RefProblem(p)
    x = np.random.default_rng(2).standard_normal(p.d).astype(np.float32)
    assert abs(oracle.objective(rp, x) - _numpy_objective(p.dense, p.y, x, p.l2, p.l1)) < 1e-7
    g, z = oracle.full_grad(rp, x, want_margins=True)
    # l2 is a float32 inside the problem descriptor
    assert np.allclose(g, _numpy_grad(p.dense, p.y, x, float(np.float32(p.l2))), rtol=2e-7, atol=1e-9)
    assert np.allclose(z, p.dense.astype(np.float64) @ x.astype(np.float64), rtol=1e-6, atol=1e-7)


def test_csr_equals_dense():
    p = _small_csr()
    pd = _densify(p)
    rs, rd = oracle.RefProblem(p), oracle.RefProblem(pd)
    rng = np.random.default_rng(5)
    x = rng.standard_normal(p.d).astype(np.float32)
    xs = (x + 0.05 * rng.standard_normal(p.d)).astype(np.float32)
    assert abs(oracle.objective(rs, x) - oracle.objective(rd, x)) < 1e-12
    assert np.array_equal(oracle.full_grad(rs, x), oracle.full_grad(rd, x))
    idx = rng.integers(0, p.n, size=16).astype(np.int32)
    a, b = oracle.vr_grad(rs, idx, x, xs), oracle.vr_grad(rd, idx, x, xs)
    assert np.allclose(a, b, rtol=1e-6, atol=1e-10)


@pytest.mark.parametrize("make", [_small_dense, _small_csr])
def test_vr_grad_structure(make):
    p = make()
    rp = oracle.RefProblem(p)
    rng = np.random.default_rng(6)
    xs = (0.3 * rng.standard_normal(p.d)).astype(np.float32)
    q = (xs + 0.1 * rng.standard_normal(p.d)).astype(np.float32)
    idx = rng.integers(0, p.n, size=8).astype(np.int32)
    # model equals snapshot: the difference vanishes identically
    assert not oracle.vr_grad(rp, idx, xs, xs).any()
    # the batch of all n points gives grad f(q) - grad f(xs)   (Assumption 1)
    all_idx = np.arange(p.n, dtype=np.int32)
    full = oracle.vr_grad(rp, all_idx, q, xs)
    gq, gs = oracle.full_grad(rp, q).astype(np.float64), oracle.full_grad(rp, xs).astype(np.float64)
    want = gq - gs                      # each term carries one float32 rounding of its own size
    assert np.allclose(full, want, rtol=0, atol=2e-7 * max(np.abs(gq).max(), np.abs(gs).max()))
    # a concatenated batch is the mean of its halves; duplicates count twice
    a = oracle.vr_grad(rp, idx[:4], q, xs).astype(np.float64)
    b = oracle.vr_grad(rp, idx[4:], q, xs).astype(np.float64)
    ab = oracle.vr_grad(rp, idx, q, xs)
    assert np.allclose(ab, 0.5 * (a + b), rtol=0, atol=2e-7 * np.abs(ab).max())
    dup = oracle.vr_grad(rp, np.array([idx[0], idx[0], idx[1]], dtype=np.int32), q, xs).astype(np.float64)
    s0 = oracle.vr_grad(rp, idx[:1], q, xs).astype(np.float64)
    s1 = oracle.vr_grad(rp, idx[1:2], q, xs).astype(np.float64)
    assert np.allclose(dup, (2 * s0 + s1) / 3, rtol=0, atol=3e-7 * np.abs(dup).max())


def test_vr_grad_brute_force_tiny():
    p = synth.dense_logistic(12, 5, seed=9, l2=0.05, l1=0.0)
    rp = oracle.RefProblem(p)
    rng = np.random.default_rng(3)
    xs = rng.standard_normal(5).astype(np.float32)
    q = rng.standard_normal(5).astype(np.float32)
    idx = np.array([3, 7, 7, 0], dtype=np.int32)
    X, y = p.dense.astype(np.float64), p.y.astype(np.float64)
    l2 = float(np.float32(p.l2))
    want = np.zeros(5)
    for i in idx:                       # grad f_i(q) - grad f_i(xs), averaged over the batch
        gq = -y[i] / (1 + np.exp(y[i] * (X[i] @ q.astype(np.float64)))) * X[i] + l2 * q
        gs = -y[i] / (1 + np.exp(y[i] * (X[i] @ xs.astype(np.float64)))) * X[i] + l2 * xs
        want += (gq - gs) / idx.size
    assert np.allclose(oracle.vr_grad(rp, idx, q, xs), want, rtol=1e-6, atol=1e-9)
