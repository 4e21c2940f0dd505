"""Pins for the oracle's sparse message format (CPU only): Section 4.2 of the paper,
32 bits for the scale plus, per nonzero coordinate, log d bits of position and b bits of value."""
import math
import os

import numpy as np
import pytest

import oracle


def _rows(path):
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            yield [f.strip() for f in line.split(";")]


def test_worked_examples(golden_dir):
    n = 0
    for d, b, codes, nnz, words in _rows(os.path.join(golden_dir, "sparse_wire_worked_examples.txt")):
        d, b, nnz = int(d), int(b), int(nnz)
        codes = np.array(codes.split(), dtype=np.int8)
        want = [int(t, 16) for t in words.split()]
        got, k = oracle.sparse_encode(codes, b)
        assert k == nnz and got[: len(want)].tolist() == want and not got[len(want):].any()
        assert oracle.sparse_decode(got, k, d, b).tolist() == codes.tolist()
        n += 1
    assert n == 4


@pytest.mark.parametrize("b", [2, 4, 8])
@pytest.mark.parametrize("d", [1, 2, 3, 17, 1000, 20958])
def test_round_trip_and_size(d, b):
    rng = np.random.default_rng(d * 10 + b)
    for density in (0.0, 0.02, 0.5, 1.0):
        codes = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=d).astype(np.int8)
        codes[rng.random(d) >= density] = 0
        words, nnz = oracle.sparse_encode(codes, b)
        assert nnz == np.count_nonzero(codes)
        pb = oracle.position_bits(d)
        assert pb == (0 if d == 1 else math.ceil(math.log2(d)))
        used = (nnz * (pb + b) + 31) // 32                    # the message is 32 + nnz*(log d + b) bits
        assert not words[used:].any()
        assert np.array_equal(oracle.sparse_decode(words, nnz, d, b), codes)
        # independent reading of the stream with Python integers: positions ascend, values match
        big = sum(int(w) << (32 * i) for i, w in enumerate(words.tolist()))
        E, prev = pb + b, -1
        for e in range(nnz):
            entry = (big >> (e * E)) & ((1 << E) - 1)
            pos, f = entry & ((1 << pb) - 1), entry >> pb
            val = f - (1 << b) if f >> (b - 1) else f
            assert pos > prev and codes[pos] == val
            prev = pos


def test_sparse_message_is_smaller_when_sparse_enough():
    d, b = 20958, 4
    dense_bits = 32 + b * d
    pb = oracle.position_bits(d)
    for nnz in (100, 2000, 4000):
        assert 32 + nnz * (pb + b) < dense_bits
    assert 32 + 5000 * (pb + b) > dense_bits          # break-even near d*b/(log d + b)
