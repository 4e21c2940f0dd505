"""Pins for the oracle's quantizer, dequantizer and wire format (CPU only).

What fixes them: the definition of dom(delta,b) and Q in Section 3.1, the scale of
Alg. 1 (delta = ||v||_inf/(2^(b-1)-1)), Lemma 5 of the supplement (unbiased,
E||Q(v)-v||^2 <= d delta^2/4), hand-worked examples, and exhaustive enumeration.
"""
import itertools
import os

import numpy as np
import pytest

import oracle


def _L(b):
    return 2 ** (b - 1) - 1


def _rows(path):
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            yield [f.strip() for f in line.split(";")]


# ------------------------------------------------------------------ worked examples
def test_quantizer_worked_examples(golden_dir):
    n = 0
    for b, v, u, codes, delta in _rows(os.path.join(golden_dir, "quantizer_worked_examples.txt")):
        v = np.array(v.split(), dtype=np.float32)
        u = np.array(u.split(), dtype=np.float32)
        k, dlt, st = oracle.quantize_given_uniforms(v, int(b), u)
        assert st == 0
        assert k.tolist() == [int(t) for t in codes.split()]
        assert dlt == np.float32(delta)
        n += 1
    assert n == 5


def test_pack_worked_examples(golden_dir):
    n = 0
    for b, codes, words in _rows(os.path.join(golden_dir, "pack_worked_examples.txt")):
        b = int(b)
        codes = np.array(codes.split(), dtype=np.int8)
        want = [int(t, 16) for t in words.split()]
        got = oracle.pack(codes, b)
        assert got.tolist() == want
        assert oracle.unpack(got, codes.size, b).tolist() == codes.tolist()
        n += 1
    assert n == 4


# ---------------------------------------------------------------------- wire format
@pytest.mark.parametrize("b", [2, 4, 8])
def test_pack_roundtrip_exhaustive(b):
    per_word = 32 // b
    values = list(range(-(2 ** (b - 1)), 2 ** (b - 1)))
    # every code value at every field position of a word, with all-ones / all-zeros neighbours
    for pos in range(per_word):
        for fill in (0, -1, values[0], values[-1]):
            for val in values:
                codes = np.full(per_word * 2 + 3, fill, dtype=np.int8)
                codes[pos] = val
                codes[per_word + pos] = val
                w = oracle.pack(codes, b)
                assert w.size == (codes.size * b + 31) // 32
                assert oracle.unpack(w, codes.size, b).tolist() == codes.tolist()
                f = (int(w[0]) >> (pos * b)) & (2 ** b - 1)
                assert f == (val & (2 ** b - 1))


@pytest.mark.parametrize("b", [2, 4, 8])
def test_pack_layout_against_numpy_bits(b):
    rng = np.random.default_rng(b)
    for d in (1, 3, 16, 17, 31, 32, 33, 1000, 1001):
        codes = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=d).astype(np.int8)
        w = oracle.pack(codes, b)
        assert w.size == oracle.packed_words(d, b) == -(-d * b // 32)
        # independent construction: bit matrix -> little-endian bytes -> uint32
        fields = (codes.astype(np.int64) & (2 ** b - 1))
        bits = ((fields[:, None] >> np.arange(b)[None, :]) & 1).astype(np.uint8).reshape(-1)
        bits = np.concatenate([bits, np.zeros(w.size * 32 - bits.size, dtype=np.uint8)])
        want = np.packbits(bits, bitorder="little").view("<u4")
        assert np.array_equal(w, want)            # includes: tail bits are zero
    # the message is 32 + b*d bits (Section 3.1): delta plus ceil(b*d/32) words cover it
    assert 32 * oracle.packed_words(1000, b) >= b * 1000 > 32 * (oracle.packed_words(1000, b) - 1)


# ------------------------------------------------------------------------ invariants
@pytest.mark.parametrize("b", [2, 3, 4, 5, 8])
def test_codes_on_grid_and_bracketing(b):
    rng = np.random.default_rng(10 + b)
    L = _L(b)
    for trial in range(20):
        d = int(rng.integers(1, 400))
        v = (rng.standard_normal(d) * 10.0 ** rng.integers(-6, 6)).astype(np.float32)
        k, delta, st = oracle.quantize(v, b, seed=trial, it=trial, worker=1)
        assert st == 0
        assert k.min() >= -(2 ** (b - 1)) and k.max() <= L
        amax = np.abs(v).max()
        assert delta == np.float32(amax / np.float32(L))
        # Q(v_i) is one of the two grid points around v_i: |Q - v| <= delta (+ rounding of t)
        t = v.astype(np.float64) * L / float(amax)
        assert np.all(k >= np.floor(t - 1e-5)) and np.all(k <= np.floor(t + 1e-5) + 1)
        q = oracle.dequantize(k, delta)
        assert np.array_equal(q, (np.float32(delta) * k.astype(np.float32)))
        assert np.all(np.abs(q.astype(np.float64) - v) <= float(delta) * (1 + 1e-5))
        # the largest coordinate sits on the end point of the grid
        i = int(np.argmax(np.abs(v)))
        assert k[i] == (L if v[i] > 0 else -L)


@pytest.mark.parametrize("b", [2, 4, 8])
def test_grid_points_are_fixed_points(b):
    L = _L(b)
    delta = np.float32(2.0 ** -5)                     # power of two: t is exact
    k0 = np.arange(-L, L + 1).astype(np.int8)
    v = delta * k0.astype(np.float32)
    for seed in range(5):
        k, dlt, _ = oracle.quantize(v, b, seed, 0, 0)
        assert dlt == delta and np.array_equal(k, k0)


def test_threshold_is_strict_and_24_bit():
    # v/delta = 0.25 exactly: up iff u < 0.25
    v = np.array([127.0, 0.25], dtype=np.float32)
    for u1, want in [(0.25 - 2.0 ** -24, 1), (0.25, 0), (0.0, 1), (1 - 2.0 ** -24, 0)]:
        k, _, _ = oracle.quantize_given_uniforms(v, 8, np.array([0.5, u1], dtype=np.float32))
        assert k[1] == want
    # p = 0 never rounds up, even with u = 0
    k, _, _ = oracle.quantize_given_uniforms(np.array([127.0, 3.0], dtype=np.float32), 8,
                                             np.zeros(2, dtype=np.float32))
    assert k.tolist() == [127, 3]


def test_degenerate_inputs():
    z = np.zeros(7, dtype=np.float32)
    k, delta, st = oracle.quantize(z, 8, 0, 0, 0)
    assert st == 0 and delta == 0 and not k.any()
    assert not oracle.dequantize(k, delta).any()
    # a scale that underflows the normal range is treated as zero
    tiny = np.array([1e-44, -3e-45], dtype=np.float32)
    k, delta, st = oracle.quantize(tiny, 8, 0, 0, 0)
    assert st == 0 and delta == 0 and not k.any()
    for bad in (np.nan, np.inf, -np.inf):
        v = np.array([1.0, bad, -2.0], dtype=np.float32)
        k, delta, st = oracle.quantize(v, 4, 0, 0, 0)
        assert st == 1 and not k.any() and not np.isfinite(delta)
    # d = 0
    k, delta, st = oracle.quantize(np.zeros(0, dtype=np.float32), 4, 0, 0, 0)
    assert k.size == 0 and delta == 0 and st == 0
    # b = 2: levels {-1, 0, 1} reachable, -2 never produced with the max-norm scale
    v = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    k, _, _ = oracle.quantize(v, 2, 1, 1, 1)
    assert set(np.unique(k).tolist()) <= {-1, 0, 1}


# --------------------------------------------------- exact distribution, d <= 8
def _enumerate(v, b):
    """All up/down outcomes of the quantizer with their probabilities.

    Outcomes are forced through the supplied uniforms (u=0: up, u=1-2^-24: down);
    probabilities are computed here in float64 from the definition, independently of
    the oracle.  A coordinate that sits on a grid point (the largest one always does)
    has a single outcome and gets u=0.5: float32 rounding of t may leave it a hair
    beside the grid point, which must not matter.
    """
    d = v.size
    L = _L(b)
    amax = float(np.abs(v).max())
    delta = amax / L
    t = v.astype(np.float64) / delta
    p = t - np.floor(t)
    on_grid = np.minimum(p, 1 - p) < 1e-5
    p = np.where(on_grid, 0.0, p)
    free = [i for i in range(d) if not on_grid[i]]
    lo, hi = np.float32(0.0), np.float32(1 - 2.0 ** -24)
    mean = np.zeros(d)
    second = 0.0
    total = 0.0
    for ups in itertools.product((0, 1), repeat=len(free)):
        u = np.full(d, 0.5, dtype=np.float32)
        pr = 1.0
        for e, i in zip(ups, free):
            u[i] = lo if e else hi
            pr *= p[i] if e else 1 - p[i]
        k, dlt, _ = oracle.quantize_given_uniforms(v, b, u)
        q = oracle.dequantize(k, dlt).astype(np.float64)
        mean += pr * q
        second += pr * np.sum((q - v) ** 2)
        total += pr
    return mean, second, total, delta, p


@pytest.mark.parametrize("b", [2, 3, 4, 8])
@pytest.mark.parametrize("d", [1, 2, 5, 8])
def test_unbiased_and_variance_by_enumeration(b, d):
    rng = np.random.default_rng(100 * b + d)
    v = rng.standard_normal(d).astype(np.float32)
    mean, second, total, delta, p = _enumerate(v, b)
    assert abs(total - 1) < 1e-12
    scale = float(np.abs(v).max())
    assert np.allclose(mean, v, rtol=0, atol=2e-6 * scale)                       # E[Q(v)] = v
    assert np.isclose(second, delta ** 2 * np.sum(p * (1 - p)), rtol=1e-4, atol=1e-12)
    assert second <= d * delta ** 2 / 4 * (1 + 1e-6)                             # Lemma 5


@pytest.mark.parametrize("b", [2, 4, 8])
def test_unbiased_monte_carlo_with_the_generator(b):
    rng = np.random.default_rng(7)
    d, T = 64, 4000
    v = rng.standard_normal(d).astype(np.float32)
    L = _L(b)
    delta = float(np.abs(v).max()) / L
    t = v.astype(np.float64) / delta
    p = t - np.floor(t)
    acc = np.zeros(d)
    err2 = 0.0
    for it in range(T):
        k, dlt, _ = oracle.quantize(v, b, seed=11, it=it, worker=2)
        q = oracle.dequantize(k, dlt).astype(np.float64)
        acc += q
        err2 += np.sum((q - v) ** 2)
    sigma = delta * np.sqrt(p * (1 - p) / T)
    assert np.all(np.abs(acc / T - v) <= 5 * sigma + 1e-6)
    expect = delta ** 2 * np.sum(p * (1 - p))
    assert abs(err2 / T - expect) < 0.1 * expect
    assert err2 / T <= d * delta ** 2 / 4


def test_error_shrinks_with_bits():
    v = np.random.default_rng(3).standard_normal(20000).astype(np.float32)
    mse = {}
    for b in (2, 4, 8):
        k, dlt, _ = oracle.quantize(v, b, 5, 0, 0)
        mse[b] = np.mean((oracle.dequantize(k, dlt).astype(np.float64) - v) ** 2)
    # per-coordinate variance delta^2 p(1-p): for b>=4 p is ~uniform => delta^2/6
    amax = float(np.abs(v).max())
    for b in (4, 8):
        assert abs(mse[b] / ((amax / _L(b)) ** 2 / 6) - 1) < 0.1
    assert mse[2] > mse[4] > mse[8]
    assert abs(mse[4] / mse[8] / (_L(8) / _L(4)) ** 2 - 1) < 0.1


def test_streams_are_independent_of_each_other():
    v = np.random.default_rng(4).standard_normal(4096).astype(np.float32)
    a, _, _ = oracle.quantize(v, 4, 1, 0, 0)
    assert np.array_equal(a, oracle.quantize(v, 4, 1, 0, 0)[0])          # reproducible
    for other in (oracle.quantize(v, 4, 2, 0, 0), oracle.quantize(v, 4, 1, 1, 0),
                  oracle.quantize(v, 4, 1, 0, 1), oracle.quantize(v, 4, 1, 0, 0, oracle.TAG_MODEL)):
        frac = np.mean(a != other[0])
        assert 0.2 < frac < 0.6       # two independent roundings differ w.p. 2p(1-p) ~ 1/3 on average
