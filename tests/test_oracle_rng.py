"""Pins for the oracle's counter-based generator and stream addressing (CPU only).

The paper says only "with probability" (Section 3.1, eq. (3)); the generator is
Philox4x32-10 from its published definition.  Pins: the published known-answer
vectors, an independent big-integer implementation written here, and statistics.
"""
import os

import numpy as np

import oracle

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox_py(ctr, key, rounds=10):
    """Philox4x32 in Python integers: an implementation independent of the C one."""
    c = [int(v) for v in ctr]
    k = [int(v) for v in key]
    for _ in range(rounds):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK, p1 & MASK, ((p0 >> 32) ^ c[3] ^ k[1]) & MASK, p0 & MASK]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return c


def word_py(seed, it, worker, tag, coord):
    out = philox_py([(coord >> 2) & MASK, it, worker, tag], [seed & MASK, (seed >> 32) & MASK])
    return out[coord & 3]


def test_known_answer_vectors(golden_dir):
    rows = 0
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        h = [int(t, 16) for t in line.split()]
        ctr, key, want = h[0:4], h[4:6], h[6:10]
        assert list(oracle.philox4x32_10(ctr, key)) == want
        assert philox_py(ctr, key) == want
        rows += 1
    assert rows == 3


def test_against_bigint_implementation():
    rng = np.random.default_rng(1)
    for _ in range(3000):
        ctr = rng.integers(0, 2**32, size=4, dtype=np.uint64)
        key = rng.integers(0, 2**32, size=2, dtype=np.uint64)
        assert list(oracle.philox4x32_10(ctr, key)) == philox_py(ctr, key)


def test_stream_addressing():
    rng = np.random.default_rng(2)
    for _ in range(2000):
        seed = int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2))
        it, worker = int(rng.integers(0, 2**32)), int(rng.integers(0, 2**32))
        tag = int(rng.integers(0, 4))
        coord = int(rng.integers(0, 2**34))
        w = oracle.random_word(seed, it, worker, tag, coord)
        assert w == word_py(seed, it, worker, tag, coord)
        u = oracle.uniform(seed, it, worker, tag, coord)
        assert u == (w >> 8) / 2.0**24
        assert 0.0 <= u < 1.0
    # neighbouring coordinates share a block; streams differ by tag/worker/iter
    a = [oracle.random_word(5, 1, 2, 0, c) for c in range(8)]
    assert a[:4] == philox_py([0, 1, 2, 0], [5, 0]) and a[4:] == philox_py([1, 1, 2, 0], [5, 0])
    assert oracle.random_word(5, 1, 2, 0, 0) != oracle.random_word(5, 1, 2, 1, 0)
    assert oracle.random_word(5, 1, 2, 0, 0) != oracle.random_word(5, 1, 3, 0, 0)
    assert oracle.random_word(5, 1, 2, 0, 0) != oracle.random_word(5, 2, 2, 0, 0)
    assert oracle.random_word(5, 1, 2, 0, 0) != oracle.random_word(5 + 2**32, 1, 2, 0, 0)


def test_uniform_statistics():
    n = 40000
    u = np.array([oracle.uniform(123, 7, 3, oracle.TAG_GRAD, c) for c in range(n)])
    assert abs(u.mean() - 0.5) < 5 * np.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 0.004
    hist, _ = np.histogram(u, bins=16, range=(0, 1))
    chi2 = ((hist - n / 16) ** 2 / (n / 16)).sum()
    assert chi2 < 50.0          # 15 dof: P(chi2 > 50) ~ 1e-5
    # serial correlation of neighbours
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.03


def test_sample_indices():
    n, B = 2000, 4096
    idx = oracle.sample_indices(n, B, 9, 4, 1)
    assert idx.min() >= 0 and idx.max() < n
    want = [(word_py(9, 4, 1, oracle.TAG_SAMPLE, j) * n) >> 32 for j in range(B)]
    assert idx.tolist() == want
    counts = np.bincount(idx, minlength=n)
    assert counts.max() <= 12            # Poisson(2.05) tail
    assert abs(idx.mean() - (n - 1) / 2) < 5 * n / np.sqrt(12 * B)
    # n = 1 and huge n stay in range
    assert oracle.sample_indices(1, 8, 0, 0, 0).tolist() == [0] * 8
    big = oracle.sample_indices(2**31 - 1, 64, 0, 0, 0)
    assert big.min() >= 0
