"""Pins for the oracle's gradient sparsifier (CPU only).

What fixes it: eq. (3) of the paper, E[beta] = alpha, phi = sum p_i, Lemma 2
(E||beta||^2 = ||alpha||_1^2 / phi at the optimal p_i), and the special case of the
budget of Section 5.1 (phi = ||alpha||_1/||alpha||_inf), where every kept coordinate
has magnitude ||alpha||_inf.
"""
import itertools

import numpy as np
import pytest

import oracle


def _probabilities(alpha, phi):
    a = np.abs(alpha.astype(np.float64))
    if phi is None:
        return a / a.max()
    return np.minimum(1.0, a * phi / a.sum())


@pytest.mark.parametrize("phi_frac", [None, 1.0, 0.5, 0.1])
@pytest.mark.parametrize("d", [1, 3, 8])
def test_moments_by_enumeration(d, phi_frac):
    rng = np.random.default_rng(17 * d)
    alpha = rng.standard_normal(d).astype(np.float32)
    if d >= 3:
        alpha[1] = 0.0                                     # p_i = 0 coordinate
    a64 = alpha.astype(np.float64)
    bound = np.abs(a64).sum() / np.abs(a64).max()          # Lemma 2: phi <= ||alpha||_1/||alpha||_inf
    phi = None if phi_frac is None else phi_frac * bound
    p = _probabilities(alpha, phi)
    eff_phi = bound if phi is None else phi
    assert abs(p.sum() - eff_phi) < 1e-9                   # phi = sum p_i
    lo, hi = np.float32(0.0), np.float32(1 - 2.0 ** -24)
    free = [i for i in range(d) if 0 < p[i] < 1 - 1e-6]
    mean, second, total = np.zeros(d), 0.0, 0.0
    for keep in itertools.product((0, 1), repeat=len(free)):
        u = np.full(d, 0.5, dtype=np.float32)
        pr = 1.0
        for e, i in zip(keep, free):
            u[i] = lo if e else hi
            pr *= p[i] if e else 1 - p[i]
        beta, nnz = oracle.sparsify_given_uniforms(alpha, u, -1.0 if phi is None else phi)
        assert nnz == np.count_nonzero(beta)
        mean += pr * beta
        second += pr * np.sum(beta.astype(np.float64) ** 2)
        total += pr
    assert abs(total - 1) < 1e-12
    assert np.allclose(mean, a64, rtol=0, atol=3e-7 * np.abs(a64).max())        # E[beta] = alpha
    assert np.isclose(second, np.abs(a64).sum() ** 2 / eff_phi, rtol=1e-5)       # Lemma 2, equality case


def test_default_budget_is_ternary_in_magnitude():
    rng = np.random.default_rng(1)
    alpha = (rng.standard_normal(5000) * np.where(rng.random(5000) < 0.1, 1.0, 0.01)).astype(np.float32)
    amax = np.abs(alpha).max()
    beta, nnz = oracle.sparsify(alpha, 3, 0, 1)
    kept = beta != 0
    assert nnz == kept.sum() and 0 < nnz < alpha.size
    assert np.all(np.sign(beta[kept]) == np.sign(alpha[kept]))
    assert np.allclose(np.abs(beta[kept]), amax, rtol=3e-7, atol=0)
    assert beta[np.argmax(np.abs(alpha))] == alpha[np.argmax(np.abs(alpha))]     # p = 1: always kept
    # expected number kept = phi = ||alpha||_1/||alpha||_inf
    phi = np.abs(alpha.astype(np.float64)).sum() / float(amax)
    assert abs(nnz - phi) < 5 * np.sqrt(phi)


def test_threshold_and_cap():
    alpha = np.array([4.0, -1.0, 0.0, 2.0], dtype=np.float32)
    # default budget: p = |alpha|/4 = [1, .25, 0, .5]
    beta, nnz = oracle.sparsify_given_uniforms(alpha, np.array([0.999, 0.25, 0.0, 0.49], dtype=np.float32))
    assert beta.tolist() == [4.0, 0.0, 0.0, 4.0] and nnz == 2
    beta, _ = oracle.sparsify_given_uniforms(alpha, np.array([0.0, 0.2499, 0.0, 0.5], dtype=np.float32))
    assert beta.tolist() == [4.0, -4.0, 0.0, 0.0]
    # caller's phi above the bound of Lemma 2: probabilities are capped at 1
    beta, nnz = oracle.sparsify_given_uniforms(alpha, np.full(4, 0.9, dtype=np.float32), phi=7.0)
    # p = min(1, |alpha|*7/7) = [1, 1, 0, 1]
    assert beta.tolist() == [4.0, -1.0, 0.0, 2.0] and nnz == 3
    # phi = 1.75: p = |alpha|/4 again (phi/||alpha||_1 = 1/4)
    beta, _ = oracle.sparsify_given_uniforms(alpha, np.array([0.5, 0.2, 0.0, 0.6], dtype=np.float32), phi=1.75)
    assert beta.tolist() == [4.0, -4.0, 0.0, 0.0]
    # all-zero vector
    beta, nnz = oracle.sparsify(np.zeros(9, dtype=np.float32), 1, 2, 3)
    assert nnz == 0 and not beta.any()


def test_monte_carlo_with_the_generator():
    rng = np.random.default_rng(2)
    d, T = 48, 4000
    alpha = rng.standard_normal(d).astype(np.float32)
    a64 = alpha.astype(np.float64)
    phi = 0.5 * np.abs(a64).sum() / np.abs(a64).max()
    p = _probabilities(alpha, phi)
    acc, kept, sq = np.zeros(d), 0, 0.0
    for it in range(T):
        beta, nnz = oracle.sparsify(alpha, 77, it, 5, phi=phi)
        acc += beta
        kept += nnz
        sq += np.sum(beta.astype(np.float64) ** 2)
    sigma = np.abs(a64) * np.sqrt((1 - p) / p / T)
    assert np.all(np.abs(acc / T - a64) <= 5 * sigma + 1e-6)
    assert abs(kept / T - phi) < 5 * np.sqrt(phi / T)
    assert abs(sq / T / (np.abs(a64).sum() ** 2 / phi) - 1) < 0.05
    # the sparsifier stream differs from the quantizer stream of the same worker
    u_s = [oracle.uniform(77, 0, 5, oracle.TAG_SPARSIFY, c) for c in range(8)]
    u_g = [oracle.uniform(77, 0, 5, oracle.TAG_GRAD, c) for c in range(8)]
    assert u_s != u_g


def test_sparsify_then_quantize_codes():
    # With the default budget the quantized message is ternary up to one rounding (b=4: 0, +-7, maybe +-6).
    rng = np.random.default_rng(4)
    alpha = rng.standard_normal(3000).astype(np.float32)
    beta, _ = oracle.sparsify(alpha, 1, 1, 1)
    k, delta, _ = oracle.quantize(beta, 4, 1, 1, 1)
    assert set(np.unique(np.abs(k)).tolist()) <= {0, 6, 7}
    assert np.mean(np.abs(k[k != 0]) == 7) > 0.99
