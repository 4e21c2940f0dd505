"""Pins for the oracle's evaluation of condition (2) / (4) of the paper (CPU only).

E_Q||Q(x)-x||^2 is pinned by exact enumeration of the quantizer's outcomes for d <= 8, by
Monte-Carlo with the generator, by Lemma 5's bound d*delta^2/4 and by its scaling with b.
"""
import itertools

import numpy as np
import pytest

import oracle


def _L(b):
    return 2 ** (b - 1) - 1


@pytest.mark.parametrize("b", [2, 3, 4, 8])
@pytest.mark.parametrize("d", [1, 4, 8])
def test_expected_error_by_enumeration(b, d):
    rng = np.random.default_rng(31 * b + d)
    v = rng.standard_normal(d).astype(np.float32)
    amax = float(np.abs(v).max())
    delta = amax / _L(b)
    t = v.astype(np.float64) / delta
    p = t - np.floor(t)
    on_grid = np.minimum(p, 1 - p) < 1e-5
    free = [i for i in range(d) if not on_grid[i]]
    total = 0.0
    for ups in itertools.product((0, 1), repeat=len(free)):
        u = np.full(d, 0.5, dtype=np.float32)
        pr = 1.0
        for e, i in zip(ups, free):
            u[i] = 0.0 if e else np.float32(1 - 2.0 ** -24)
            pr *= p[i] if e else 1 - p[i]
        k, dl, _ = oracle.quantize_given_uniforms(v, b, u)
        total += pr * np.sum((oracle.dequantize(k, dl).astype(np.float64) - v) ** 2)
    got = oracle.expected_sq_error(v, b)
    # a coordinate on a grid point may sit one float32 ulp beside it: p(1-p) <= 2^-16 there
    assert abs(got - total) <= 2e-4 * total + 2e-5 * d * delta ** 2
    assert got <= d * delta ** 2 / 4 * (1 + 1e-6)


def test_expected_error_monte_carlo_and_scaling():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(2000).astype(np.float32)
    errs = {}
    for b in (2, 4, 8):
        errs[b] = oracle.expected_sq_error(x, b)
        mc = np.mean([np.sum((oracle.dequantize(*oracle.quantize(x, b, 3, it, 0)[:2]).astype(np.float64) - x) ** 2)
                      for it in range(200)])
        assert abs(mc / errs[b] - 1) < 0.05
    assert errs[2] > errs[4] > errs[8]
    assert abs(errs[4] / errs[8] / (_L(8) / _L(4)) ** 2 - 1) < 0.1
    assert oracle.expected_sq_error(np.zeros(5, dtype=np.float32), 8) == 0.0
    tiny = np.full(4, 1e-44, dtype=np.float32)           # degenerate scale: everything rounds to zero
    assert np.isclose(oracle.expected_sq_error(tiny, 8), np.sum(tiny.astype(np.float64) ** 2))


def test_distance_and_bx_choice():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(500).astype(np.float32)
    xs = (x + 0.05 * rng.standard_normal(500)).astype(np.float32)
    r = oracle.sq_distance(x, xs)
    assert np.isclose(r, np.sum((x.astype(np.float64) - xs) ** 2))
    e = {b: oracle.expected_sq_error(x, b) for b in (2, 4, 8)}
    # a larger mu admits fewer bits (Section 4.1); a tiny mu admits none of the candidates
    assert oracle.smallest_bx(x, xs, mu=1.01 * e[2] / r) == 2
    assert oracle.smallest_bx(x, xs, mu=1.01 * e[4] / r) == 4
    assert oracle.smallest_bx(x, xs, mu=1.01 * e[8] / r) == 8
    assert oracle.smallest_bx(x, xs, mu=0.5 * e[8] / r, candidates=(2, 4, 8)) == 32
    # every width from 2 to 16 is a candidate by default (Section 5.2 searches b_x over all of them):
    # one more bit divides the expected error by about four
    assert oracle.smallest_bx(x, xs, mu=0.5 * e[8] / r) == 9
    assert oracle.smallest_bx(x, xs, mu=1.01 * oracle.expected_sq_error(x, 11) / r) == 11
    assert oracle.smallest_bx(x, xs, mu=1e-3 * oracle.expected_sq_error(x, 16) / r) == 32
    k, dl, _ = oracle.quantize(x, 8, 1, 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    realised, dist = oracle.mu_terms(k, dl, x, xs)
    assert np.isclose(dist, r) and abs(realised / e[8] - 1) < 0.2
