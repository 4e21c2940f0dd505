"""Pins for the oracle's unquantized modes (CPU only): the comparison algorithms of Section 5.1.

AsyFPG / Acc-AsyFPG remove double quantization; QSVRG quantizes gradients only.  With the
quantizers switched off the loop is plain mini-batch proximal SVRG, which is checked against a
float64 implementation written here on the same index streams.
"""
import numpy as np

import oracle
from oracle import algorithms as alg
import synth
from test_oracle_algorithms import _full_precision_svrg, _obj64


def test_master_update_full_matches_code_path():
    rng = np.random.default_rng(0)
    M, d = 5, 300
    codes = rng.integers(-128, 128, size=(M, d)).astype(np.int8)
    g = rng.standard_normal(d).astype(np.float32)
    x0, y0, xs = (rng.standard_normal(d).astype(np.float32) for _ in range(3))
    for acc in (False, True):
        xa, xb, ya, yb = x0.copy(), x0.copy(), y0.copy(), y0.copy()
        sa, sb = np.zeros(d, dtype=np.float32), np.zeros(d, dtype=np.float32)
        kw = dict(eta=0.01, theta=0.5, l1=0.02)
        oracle.master_update(codes, np.ones(M, dtype=np.float32), 0.2, g, xa, ya if acc else None, xs, sa if acc else None, **kw)
        oracle.master_update_full(codes.astype(np.float32), 0.2, g, xb, yb if acc else None, xs, sb if acc else None, **kw)
        assert np.array_equal(xa, xb) and np.array_equal(ya, yb) and np.array_equal(sa, sb)


def test_unquantized_run_is_plain_prox_svrg():
    p = synth.dense_logistic(300, 40, seed=1, l2=1e-3, l1=1e-4)
    M, B, m, S, lr = 3, 8, 30, 2, 0.5
    tr = alg.run(p, "asylpg", M, B, 32, 32, m, S, lr, seed=5)
    ref = _full_precision_svrg(p, M, B, m, S, lr, seed=5)
    assert np.linalg.norm(tr.x_snap - ref) < 1e-5 * np.linalg.norm(ref)
    assert abs(tr.objectives[-1] - _obj64(p, ref)) < 1e-6
    assert tr.bits_up == S * m * M * 32 * p.d
    assert tr.bits_down == S * (1 + (m - 1) * 32 * p.d)


def test_bits_saved_by_quantization():
    p = synth.dense_logistic(300, 40, seed=1, l2=1e-3)
    M, B, m, S, lr = 3, 8, 30, 2, 0.5
    fp = alg.run(p, "asylpg", M, B, 32, 32, m, S, lr, seed=5)
    qsvrg = alg.run(p, "asylpg", M, B, 32, 8, m, S, lr, seed=5)          # gradients quantized only
    lp = alg.run(p, "asylpg", M, B, 8, 8, m, S, lr, seed=5)              # double quantization
    d = p.d
    assert qsvrg.bits_up == lp.bits_up == S * m * M * (32 + 8 * d)
    assert qsvrg.bits_down == fp.bits_down > lp.bits_down
    total = lambda t: t.bits_up + M * t.bits_down
    assert total(lp) < total(qsvrg) < total(fp)
    assert abs(total(fp) / total(lp) - 32 * d / (32 + 8 * d)) < 0.02 * 4           # close to the per-message ratio
    for t in (qsvrg, lp):                                                            # similar convergence (Section 5.1)
        assert abs(t.objectives[-1] - fp.objectives[-1]) < 0.01 * fp.objectives[-1]


def test_accelerated_unquantized():
    p = synth.dense_logistic(200, 30, seed=4, l2=1e-3)
    a = alg.run(p, "acc", 2, 8, 32, 32, 15, 3, 0.2, seed=2)
    b = alg.run(p, "acc", 2, 8, 8, 8, 15, 3, 0.2, seed=2)
    assert a.objectives[-1] < a.objectives[0]
    assert abs(a.objectives[-1] - b.objectives[-1]) < 0.01 * a.objectives[-1]
    assert a.bits_up == 3 * 15 * 2 * 32 * p.d
