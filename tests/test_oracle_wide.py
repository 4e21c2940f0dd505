"""Pins for the oracle's quantizer and wire format at any width 2 <= b <= 16 (CPU only).

The model-precision study of Section 5.2 varies b_x from 2 to 11, so fields no longer divide the
32-bit words.  What fixes the format: hand-worked examples, the row read as one big integer
(a formulation that shares nothing with the oracle's word loop), agreement with the 2/4/8-bit
format, exhaustive round trips; the quantizer itself is pinned by Section 3.1's grid rules.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import algorithms

WIDTHS = list(range(2, 17))


def _rows(path):
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            yield [f.strip() for f in line.split(";")]


def test_pack_wide_worked_examples(golden_dir):
    n = 0
    for b, codes, words in _rows(os.path.join(golden_dir, "pack_wide_worked_examples.txt")):
        b = int(b)
        codes = np.array(codes.split(), dtype=np.int32)
        got = oracle.pack_wide(codes, b)
        assert got.tolist() == [int(t, 16) for t in words.split()]
        assert oracle.unpack_wide(got, codes.size, b).tolist() == codes.tolist()
        n += 1
    assert n == 4


@pytest.mark.parametrize("b", WIDTHS)
def test_pack_wide_is_one_little_endian_bit_string(b):
    rng = np.random.default_rng(100 + b)
    for d in (1, 2, 31, 32, 33, 97, 1000):
        codes = rng.integers(-(1 << (b - 1)), 1 << (b - 1), size=d).astype(np.int32)
        big = 0
        for i, k in enumerate(codes.tolist()):
            big |= (k & ((1 << b) - 1)) << (i * b)
        nw = (d * b + 31) // 32
        want = [(big >> (32 * w)) & 0xFFFFFFFF for w in range(nw)]
        got = oracle.pack_wide(codes, b)
        assert got.size == nw and got.tolist() == want
        assert oracle.unpack_wide(got, d, b).tolist() == codes.tolist()


@pytest.mark.parametrize("b", [2, 4, 8])
def test_wide_format_agrees_with_the_byte_aligned_one(b):
    rng = np.random.default_rng(b)
    codes = rng.integers(-(1 << (b - 1)), 1 << (b - 1), size=777).astype(np.int8)
    assert oracle.pack_wide(codes.astype(np.int32), b).tolist() == oracle.pack(codes, b).tolist()
    assert oracle.unpack_wide(oracle.pack(codes, b), codes.size, b).tolist() == codes.tolist()


@pytest.mark.parametrize("b", [3, 5, 7, 11, 13])
def test_unpack_wide_every_value_at_every_offset(b):
    # every code value in a field that starts at every possible bit offset of a word, neighbours all ones / all zeros
    values = np.arange(-(1 << (b - 1)), 1 << (b - 1), dtype=np.int32)
    step = max(1, values.size // 64)
    for pos in range(32):                      # field `pos` starts at bit (pos*b) % 32; b odd => all 32 offsets occur
        for fill in (0, -1):
            for v in values[::step].tolist() + [int(values[-1])]:
                codes = np.full(34, fill, dtype=np.int32)
                codes[pos] = v
                w = oracle.pack_wide(codes, b)
                assert oracle.unpack_wide(w, codes.size, b).tolist() == codes.tolist()


@pytest.mark.parametrize("b", [2, 3, 4, 5, 8])
def test_quantize_wide_equals_the_narrow_quantizer(b):
    rng = np.random.default_rng(7 * b)
    v = rng.standard_normal(501).astype(np.float32)
    k8, d8, s8 = oracle.quantize(v, b, 5, 9, 3, oracle.TAG_GRAD)
    k32, d32, s32 = oracle.quantize_wide(v, b, 5, 9, 3, oracle.TAG_GRAD)
    assert k32.tolist() == k8.astype(np.int32).tolist() and d8 == d32 and s8 == s32


@pytest.mark.parametrize("b", [9, 11, 16])
def test_quantize_wide_grid_rules(b):
    # Section 3.1: the result is one of the two grid points that bracket v_i; the largest
    # coordinate sits on the last grid point; the error is below one grid step
    rng = np.random.default_rng(b)
    v = (rng.standard_normal(4000) * 0.3).astype(np.float32)
    L = 2 ** (b - 1) - 1
    k, delta, st = oracle.quantize_wide(v, b, 11, 4, 2, oracle.TAG_MODEL)
    assert st == 0
    amax = np.abs(v).max()
    assert delta == np.float32(amax / np.float32(L))
    t = v.astype(np.float64) * (L / float(amax))
    assert np.all(k >= np.floor(t) - 1e-3) and np.all(k <= np.floor(t) + 1 + 1e-3)
    assert abs(int(k[np.argmax(np.abs(v))])) == L
    assert k.min() >= -L - 1 and k.max() <= L
    q = oracle.dequantize_wide(k, delta)
    assert np.max(np.abs(q - v)) <= float(delta) * (1 + 1e-5)
    # both neighbours occur, with a frequency that matches the fractional parts (unbiased rounding)
    up = k - np.floor(t)
    frac = t - np.floor(t)
    assert abs(up.mean() - frac.mean()) < 5 * 0.5 / np.sqrt(v.size)


def test_quantize_wide_error_shrinks_by_four_per_two_bits():
    # delta halves with every extra bit, E||Q(v)-v||^2 = delta^2 sum p(1-p): a factor ~4 per bit
    rng = np.random.default_rng(1)
    v = rng.standard_normal(20000).astype(np.float32)
    err = {}
    for b in (6, 8, 10, 12):
        k, delta, _ = oracle.quantize_wide(v, b, 3, 0, 0, oracle.TAG_GRAD)
        err[b] = float(np.sum((oracle.dequantize_wide(k, delta).astype(np.float64) - v) ** 2))
    for b in (6, 8, 10):
        assert 12.0 < err[b] / err[b + 2] < 21.0          # (L_{b+2}/L_b)^2 ~ 16


@pytest.mark.parametrize("b_x", [3, 5, 11])
def test_model_message_any_width(b_x):
    rng = np.random.default_rng(b_x)
    d = 333
    x = rng.standard_normal(d).astype(np.float32)
    xs = np.zeros(d, dtype=np.float32)
    q, words, dx, bits = algorithms.model_message(x, xs, b_x, 1, 2)
    assert bits == 32 + b_x * d and words.size == (d * b_x + 31) // 32
    k = np.rint(q / dx).astype(np.int64)
    assert np.allclose(k * float(dx), q, rtol=1e-6, atol=0)
    assert np.max(np.abs(q - x)) <= float(dx) * (1 + 1e-5)
    assert oracle.unpack_wide(words, d, b_x).tolist() == k.tolist()
