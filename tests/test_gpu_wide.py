"""GPU parity for model messages of any width 2 <= b_x <= 16 (model-precision study, Section 5.2):
quantize+pack, decode+sum, the worker's decode of the model, the master's re-quantization and
whole runs, all against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle import algorithms as alg
from gpu_util import dev, host, words

pytestmark = pytest.mark.gpu

WIDE = [3, 5, 6, 7, 9, 10, 11, 12, 13, 16]


@pytest.fixture(scope="module")
def dq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1805_10111_amd as dq
    return dq


@pytest.mark.parametrize("b", WIDE)
@pytest.mark.parametrize("d", [1, 31, 32, 33, 1000, 4096, 20958, 70001])
def test_quantize_pack_any_width_bit_exact(dq, d, b):
    v = synth.mixture_vector(d, seed=17 * d + b)
    seed, it, worker = 0xFEDCBA9876543210, 5, 2
    nw = dq.packed_words(d, b)
    packed = torch.full((nw + 4,), -1, dtype=torch.int32, device="cuda")
    absmax = torch.zeros(1, device="cuda")
    delta = torch.zeros(1, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    dq.dq_quantize_pack(dev(v), b, absmax, False, seed, it, dq.TAG_MODEL, worker, packed, delta, status)
    k, dlt, st = oracle.quantize_wide(v, b, seed, it, worker, oracle.TAG_MODEL)
    assert host(delta)[0] == dlt and host(status)[0] == st == 0
    assert np.array_equal(words(packed)[:nw], oracle.pack_wide(k, b))
    assert np.all(words(packed)[nw:] == 0xFFFFFFFF)          # nothing written past the row


def test_quantize_pack_any_width_rows(dq):
    M, d, b = 5, 1003, 11
    ld = 1004
    rng = np.random.default_rng(3)
    buf = np.zeros((M, ld), dtype=np.float32)
    buf[:, :d] = rng.standard_normal((M, d)).astype(np.float32)
    buf[2, :d] = 0.0                                          # an all-zero row: delta 0, codes 0
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    absmax = torch.zeros(M, device="cuda")
    delta = torch.zeros(M, device="cuda")
    dq.dq_quantize_pack(dev(buf)[:, :d], b, absmax, False, 8, 1, dq.TAG_GRAD, 10, packed, delta, None)
    for m in range(M):
        k, dlt, _ = oracle.quantize_wide(buf[m, :d], b, 8, 1, 10 + m, oracle.TAG_GRAD)
        assert host(delta)[m] == dlt
        assert np.array_equal(words(packed)[m, :nw], oracle.pack_wide(k, b))


@pytest.mark.parametrize("b", [3, 5, 11, 16])
@pytest.mark.parametrize("M,d", [(1, 33), (4, 1000), (16, 4099)])
def test_unpack_dequant_sum_any_width_bit_exact(dq, b, M, d):
    rng = np.random.default_rng(b * 100 + M)
    k = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d)).astype(np.int32)
    delta = (rng.random(M) * 1e-2).astype(np.float32)
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    pw = np.zeros((M, ldw), dtype=np.uint32)
    for m in range(M):
        pw[m, :nw] = oracle.pack_wide(k[m], b)
    scale = np.float32(1.0 / M)
    out = torch.zeros(d, device="cuda")
    dq.dq_unpack_dequant_sum(dev(pw.view(np.int32)), dev(delta), d, b, float(scale), out)
    # fmaf(delta, k, acc) in float32 == the double-precision result rounded once (24 + 16 bit product is exact in double)
    acc32 = np.zeros(d, dtype=np.float32)
    for m in range(M):
        acc32 = (delta[m].astype(np.float64) * k[m].astype(np.float64) + acc32.astype(np.float64)).astype(np.float32)
    want = scale * acc32
    assert np.array_equal(host(out).view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("b", [3, 5, 7])
def test_pack_unpack_int8_any_width(dq, b):
    M, d = 3, 1001
    ld = 1008
    rng = np.random.default_rng(b)
    k = np.zeros((M, ld), dtype=np.int8)
    k[:, :d] = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d))
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    dq.dq_pack(dev(k)[:, :d], d, b, packed)
    for m in range(M):
        assert np.array_equal(words(packed)[m, :nw], oracle.pack_wide(k[m, :d].astype(np.int32), b))
    back = torch.zeros((M, ld), dtype=torch.int8, device="cuda")[:, :d]
    dq.dq_unpack(packed, d, b, back)
    assert np.array_equal(host(back), k[:, :d])


def _model_wide(d, b_x, x_snap, seed):
    rng = np.random.default_rng(seed)
    x = (x_snap + 0.05 * rng.standard_normal(d)).astype(np.float32)
    k, dx, _ = oracle.quantize_wide(x, b_x, 3, 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    return oracle.pack_wide(k, b_x), dx, oracle.dequantize_wide(k, dx)


@pytest.mark.parametrize("b_x", [3, 5, 11])
@pytest.mark.parametrize("layout", ["dense", "csr"])
def test_vr_grad_decodes_any_model_width(dq, layout, b_x):
    if layout == "dense":
        n, d, M, B = 300, 1027, 3, 9
        p = synth.dense_logistic(n, d, seed=4, l2=1e-3)
        lda = (d + 3) // 4 * 4
        Xp = np.zeros((n, lda), dtype=np.float32)
        Xp[:, :d] = p.dense
        P = dq.DeviceProblem(n=n, d=d, y=dev(p.y), l2=p.l2, l1=p.l1, dense=dev(Xp)[:, :d])
    else:
        n, d, M, B = 500, 3001, 4, 12
        p = synth.sparse_text_logistic(n, d, mean_nnz=20.0, seed=2)
        P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    rng = np.random.default_rng(b_x)
    x_snap = (0.2 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, q = _model_wide(d, b_x, x_snap, seed=b_x + 1)
    idx = np.stack([oracle.sample_indices(n, B, 11, 2, w) for w in range(M)])
    ld = (d + 3) // 4 * 4
    alpha = torch.zeros((M, ld), device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    dq.dq_vr_grad(P, dev(idx), M, B, dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), b_x, False,
                  dev(x_snap), None, alpha, amax, None, ws)
    for w in range(M):
        want = oracle.vr_grad(rp, idx[w], q, x_snap).astype(np.float64)
        got = host(alpha)[w].astype(np.float64)
        assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()


@pytest.mark.parametrize("acc", [False, True])
@pytest.mark.parametrize("bx", [3, 11])
@pytest.mark.parametrize("M,d", [(4, 1000), (3, 4099), (2, 40001)])
def test_master_step_any_model_width(dq, acc, bx, M, d):
    b = 8
    rng = np.random.default_rng(M + d + bx)
    k = rng.integers(-128, 128, size=(M, d)).astype(np.int8)
    delta = (rng.random(M) * 1e-2).astype(np.float32)
    nw = (d * b + 31) // 32
    ldw = (nw + 3) // 4 * 4
    pw = np.zeros((M, ldw), dtype=np.uint32)
    for m in range(M):
        pw[m, :nw] = oracle.pack(k[m], b)
    g = rng.standard_normal(d).astype(np.float32) * np.float32(0.1)
    x0, xs, y0, sum0 = (rng.standard_normal(d).astype(np.float32) for _ in range(4))
    eta, theta, l1 = np.float32(0.3), np.float32(0.4), np.float32(0.05)
    scale = np.float32(1.0 / M)
    seed, it = 77, 4
    x_ref, y_ref, s_ref = x0.copy(), y0.copy(), sum0.copy()
    if acc:
        oracle.master_update(k, delta, scale, g, x_ref, y_ref, xs, s_ref, eta=eta, theta=theta, l1=l1)
    else:
        oracle.master_update(k, delta, scale, g, x_ref, eta=eta, l1=l1)
    kx, dx, _ = oracle.quantize_wide(x_ref, bx, seed, it, oracle.MASTER_ID, oracle.TAG_MODEL)
    x, y, xsum = dev(x0), dev(y0), dev(sum0)
    nwx = dq.packed_words(d, bx)
    xq = torch.full((nwx + 4,), -1, dtype=torch.int32, device="cuda")
    dxo = torch.zeros(1, device="cuda")
    amx = torch.zeros(1, device="cuda")
    dq.dq_master_step(dev(pw.view(np.int32)), dev(delta), M, b, float(scale), dev(g), x, y if acc else None,
                      dev(xs), xsum if acc else None, float(eta), float(theta), float(l1), bx, seed, it, xq, dxo, amx)
    assert np.array_equal(host(x).view(np.uint32), x_ref.view(np.uint32))
    assert host(dxo)[0] == dx and host(amx)[0] == oracle.absmax(x_ref)
    assert np.array_equal(words(xq)[:nwx], oracle.pack_wide(kx, bx))
    assert np.all(words(xq)[nwx:] == 0xFFFFFFFF)


@pytest.mark.parametrize("algo,b_x", [("asylpg", 5), ("asylpg", 11), ("acc", 6), ("sparse", 3)])
def test_free_run_any_model_width(dq, algo, b_x):
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    cfg = synth.CONFIGS["C1"]
    p = synth.make_problem(cfg, n=600, d=204)
    m, S, b = 10, 2, 8 if algo != "sparse" else 4
    tr = DoubleQuantTrainer(dq.DeviceProblem.from_host(p), algo, cfg.M, cfg.B, b_x, b, m, cfg.lr, seed=6)
    log = tr.run(S)
    ref = alg.run(p, algo, cfg.M, cfg.B, b_x, b, m, S, cfg.lr, seed=6)
    for a, r in zip(log.objectives, ref.objectives):
        assert abs(a - r) <= 1e-5 * abs(r)
    assert log.bits_down == ref.bits_down


def test_mu_terms_any_width(dq):
    rng = np.random.default_rng(0)
    d = 3000
    x = rng.standard_normal(d).astype(np.float32)
    xs = (x + 0.01 * rng.standard_normal(d)).astype(np.float32)
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    prev = None
    for b in (3, 5, 9, 11, 16):
        dq.dq_mu_terms(dev(x), dev(xs), b, out)
        e, r = host(out)
        assert abs(e - oracle.expected_sq_error(x, b)) <= 1e-9 * e
        assert abs(r - oracle.sq_distance(x, xs)) <= 1e-9 * r
        assert prev is None or e < prev
        prev = e


def test_mu_sweep_reproduces_the_trend_of_the_model_precision_study(dq):
    """Section 5.2 (right half of Table 1): a larger mu admits a smaller b_x; each extra bit divides the mu that
    condition (2) needs by about four; and the bits sent per epoch grow with b_x."""
    from paper_1805_10111_amd.compare import mu_sweep
    cfg = synth.CONFIGS["C1"]
    p = synth.make_problem(cfg, n=600, d=200)
    res = mu_sweep(cfg, p, widths=[3, 4, 5, 6, 8, 10], epochs=2, threshold=0.0, b=8, m=10, seed=1)
    rows = res["per_width"]
    need = [rows[w]["mu_needed_median"] for w in (3, 4, 5, 6, 8, 10)]
    assert all(a > b for a, b in zip(need, need[1:]))
    assert 8.0 < rows[4]["mu_needed_median"] / rows[6]["mu_needed_median"] < 32.0      # two bits: about 16x
    bits = [rows[w]["bits_total"] for w in (3, 4, 5, 6, 8, 10)]
    assert all(a < b for a, b in zip(bits, bits[1:]))
    ch = res["smallest_width_for_mu"]
    picked = [ch[k] for k in sorted(ch, key=float) if ch[k] is not None]
    assert picked == sorted(picked, reverse=True)                  # larger mu, smaller (or equal) width
