"""GPU parity: master step, momentum epoch boundary, index sampling and sparsifier versus the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, words

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1805_10111_amd as dq
    return dq


def _messages(M, d, b, seed):
    rng = np.random.default_rng(seed)
    k = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d)).astype(np.int8)
    delta = (rng.random(M) * 1e-2).astype(np.float32)
    nw = (d * b + 31) // 32
    ldw = (nw + 3) // 4 * 4
    pw = np.zeros((M, ldw), dtype=np.uint32)
    for m in range(M):
        pw[m, :nw] = oracle.pack(k[m], b)
    return k, delta, pw


@pytest.mark.parametrize("acc", [False, True])
@pytest.mark.parametrize("b,bx", [(8, 8), (4, 8), (2, 4), (8, 2)])
@pytest.mark.parametrize("M,d", [(1, 5), (4, 1000), (8, 20958), (32, 4096), (3, 4099), (2, 8192), (2, 8193), (2, 16400), (2, 40001),
                                 (45, 4100), (70, 333), (41, 9000), (3, 9999), (2, 8194)])
def test_master_step_bit_exact(dq, acc, b, bx, M, d):
    k, delta, pw = _messages(M, d, b, seed=M * 7 + d + b)
    rng = np.random.default_rng(d)
    g = rng.standard_normal(d).astype(np.float32) * np.float32(0.1)
    x0 = rng.standard_normal(d).astype(np.float32)
    xs = rng.standard_normal(d).astype(np.float32)
    y0 = rng.standard_normal(d).astype(np.float32)
    sum0 = rng.standard_normal(d).astype(np.float32)
    eta, theta, l1 = np.float32(0.3), np.float32(0.4), np.float32(0.05)
    scale = np.float32(1.0 / M)
    seed, it = 99, 12
    # oracle
    x_ref, y_ref, s_ref = x0.copy(), y0.copy(), sum0.copy()
    if acc:
        oracle.master_update(k, delta, scale, g, x_ref, y_ref, xs, s_ref, eta=eta, theta=theta, l1=l1)
    else:
        oracle.master_update(k, delta, scale, g, x_ref, eta=eta, l1=l1)
    kx, dx, _ = oracle.quantize(x_ref, bx, seed, it, oracle.MASTER_ID, oracle.TAG_MODEL)
    # GPU
    x, y, xsum = dev(x0), dev(y0), dev(sum0)
    nwx = dq.packed_words(d, bx)
    xq = torch.full((nwx + 4,), -1, dtype=torch.int32, device="cuda")
    dxo = torch.zeros(1, device="cuda")
    amx = torch.zeros(1, device="cuda")
    dq.dq_master_step(dev(pw.view(np.int32)), dev(delta), M, b, float(scale), dev(g), x, y if acc else None,
                      dev(xs), xsum if acc else None, float(eta), float(theta), float(l1), bx, seed, it, xq, dxo, amx)
    assert np.array_equal(host(x).view(np.uint32), x_ref.view(np.uint32))
    if acc:
        assert np.array_equal(host(y).view(np.uint32), y_ref.view(np.uint32))
        assert np.array_equal(host(xsum).view(np.uint32), s_ref.view(np.uint32))
    else:
        assert np.array_equal(host(y), y0) and np.array_equal(host(xsum), sum0)
    assert host(amx)[0] == oracle.absmax(x_ref)
    assert host(dxo)[0] == dx
    assert np.array_equal(words(xq)[:nwx], oracle.pack(kx, bx))
    assert np.all(words(xq)[nwx:] == 0xFFFFFFFF)


def test_master_step_full_precision_modes(dq):
    """b = 32 / b_x = 32: the unquantized comparison algorithms of Section 5.1 through the same kernels."""
    M, d = 3, 1000
    rng = np.random.default_rng(0)
    grads = rng.standard_normal((M, d)).astype(np.float32)
    g = rng.standard_normal(d).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    x = dev(x0)
    xq = torch.zeros(d, dtype=torch.float32, device="cuda")
    dxo, amx = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
    dq.dq_master_step(dev(grads).view(torch.int32), None, M, 32, float(np.float32(1 / 3)), dev(g), x, None, None, None,
                      0.25, 0.0, 0.0, 32, 0, 0, xq.view(torch.int32), dxo, amx)
    acc = np.zeros(d, dtype=np.float32)
    for m in range(M):
        acc = acc + grads[m]
    want = x0 - np.float32(0.25) * (np.float32(1 / 3) * acc + g)
    assert np.array_equal(host(x), want)
    assert np.array_equal(host(xq), want) and host(dxo)[0] == 1.0


def test_acc_epoch_boundary(dq):
    d = 4099
    rng = np.random.default_rng(1)
    y, xs, xsum = (rng.standard_normal(d).astype(np.float32) for _ in range(3))
    out = torch.zeros(d, device="cuda")
    dq.dq_acc_mix(dev(y), dev(xs), float(np.float32(2 / 3)), out)
    assert np.array_equal(host(out), oracle.acc_mix(y, xs, np.float32(2 / 3)))
    dq.dq_acc_mix(dev(xs), dev(xs), 0.5, out)
    assert np.array_equal(host(out).view(np.uint32), xs.view(np.uint32))       # flag-bit case: bitwise snapshot
    dq.dq_acc_snapshot(dev(xsum), 25, out)
    assert np.array_equal(host(out), oracle.acc_snapshot(xsum, 25))


@pytest.mark.parametrize("n,M,B", [(2000, 4, 16), (72000, 16, 64), (200000, 32, 256), (1, 2, 5), (2**31 - 1, 2, 300)])
def test_sample_indices_bit_exact(dq, n, M, B):
    idx = torch.full((M, B), -1, dtype=torch.int32, device="cuda")
    dq.dq_sample_indices(n, M, B, 1234, 77, 5, idx)
    got = host(idx)
    for m in range(M):
        assert np.array_equal(got[m], oracle.sample_indices(n, B, 1234, 77, 5 + m))


@pytest.mark.parametrize("budget", [None, 0.5, 3.0])
@pytest.mark.parametrize("M,d", [(1, 7), (4, 1000), (3, 20958)])
def test_sparsify_bit_exact(dq, budget, M, d):
    rng = np.random.default_rng(d + M)
    alpha = (rng.standard_normal((M, d)) * np.where(rng.random((M, d)) < 0.1, 1.0, 0.01)).astype(np.float32)
    alpha[:, ::7] = 0.0
    ld = (d + 3) // 4 * 4
    abuf = np.zeros((M, ld), dtype=np.float32)
    abuf[:, :d] = alpha
    phi = None
    if budget is not None:
        phi = np.array([budget * np.abs(alpha[m]).sum() / np.abs(alpha[m]).max() for m in range(M)], dtype=np.float32)
    beta = torch.full((M, ld), 9.0, device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    nnz = torch.zeros(M, dtype=torch.int32, device="cuda")
    dq.dq_sparsify(dev(abuf)[:, :d], None if phi is None else dev(phi), 31, 4, 2, beta, amax, nnz)
    for m in range(M):
        want, kept = oracle.sparsify(alpha[m], 31, 4, 2 + m, phi=-1.0 if phi is None else float(phi[m]))
        assert np.array_equal(host(beta)[m].view(np.uint32), want.view(np.uint32))
        assert host(nnz)[m] == kept
        assert host(amax)[m] == oracle.absmax(want)


def test_master_invalid_arguments(dq):
    d = 64
    z = torch.zeros(d, device="cuda")
    p = torch.zeros(16, dtype=torch.int32, device="cuda")
    one = torch.zeros(1, device="cuda")
    with pytest.raises(dq.DqError) as e:
        dq.dq_master_step(p, one, 1, 3, 1.0, z, z.clone(), None, None, None, 0.1, 0.0, 0.0, 8, 0, 0, p.clone(), one, one.clone())
    assert e.value.code == dq.ERR_UNSUPPORTED
    with pytest.raises(dq.DqError) as e:
        dq.dq_master_step(p, one, 1, 8, 1.0, z, z.clone(), z.clone(), None, None, 0.1, 0.0, 0.0, 8, 0, 0, p.clone(), one, one.clone())
    assert e.value.code == dq.ERR_INVALID_ARG          # momentum update without a snapshot


@pytest.mark.parametrize("b", [2, 4, 8])
@pytest.mark.parametrize("d", [1, 1000, 20958, 100003])
def test_mu_terms(dq, b, d):
    rng = np.random.default_rng(d + b)
    x = rng.standard_normal(d).astype(np.float32)
    xs = (x + 0.05 * rng.standard_normal(d)).astype(np.float32)
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    dq.dq_mu_terms(dev(x), dev(xs), b, out)
    e, r = host(out)
    assert abs(e - oracle.expected_sq_error(x, b)) <= 1e-10 * oracle.expected_sq_error(x, b) + 1e-300
    assert abs(r - oracle.sq_distance(x, xs)) <= 1e-10 * oracle.sq_distance(x, xs)


def test_mu_terms_degenerate_and_bx_choice(dq):
    from paper_1805_10111_amd.driver import smallest_bx
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    z = np.zeros(50, dtype=np.float32)
    dq.dq_mu_terms(dev(z), dev(z), 8, out)
    assert host(out).tolist() == [0.0, 0.0]
    tiny = np.full(7, 1e-44, dtype=np.float32)
    dq.dq_mu_terms(dev(tiny), dev(z[:7]), 8, out)
    assert np.isclose(host(out)[0], oracle.expected_sq_error(tiny, 8), rtol=1e-12)
    rng = np.random.default_rng(3)
    x = rng.standard_normal(3000).astype(np.float32)
    xs = (x + 0.02 * rng.standard_normal(3000)).astype(np.float32)
    for mu in (1e-6, 1e-3, 0.05, 1.0, 100.0):
        assert smallest_bx(dev(x), dev(xs), mu) == oracle.smallest_bx(x, xs, mu)
    with pytest.raises(dq.DqError):
        dq.dq_mu_terms(dev(x), dev(xs), 17, out)


@pytest.mark.parametrize("acc", [False, True])
@pytest.mark.parametrize("b,bx", [(8, 8), (4, 8), (2, 4), (8, 11)])
@pytest.mark.parametrize("M,d", [(1, 5), (4, 1000), (9, 4099), (32, 4096), (2, 40001), (19, 333), (45, 4100)])
def test_master_step_each_bit_exact(dq, acc, b, bx, M, d):
    """One update per received gradient (Alg. 1, master (ii) applied message by message)."""
    k, delta, pw = _messages(M, d, b, seed=M * 5 + d + b)
    rng = np.random.default_rng(d + 1)
    g = rng.standard_normal(d).astype(np.float32) * np.float32(0.1)
    x0, xs, y0, sum0 = (rng.standard_normal(d).astype(np.float32) for _ in range(4))
    eta, theta, l1 = np.float32(0.05), np.float32(0.4), np.float32(0.05)
    seed, it = 31, 2
    x_ref, y_ref, s_ref = x0.copy(), y0.copy(), sum0.copy()
    if acc:
        oracle.master_update_each(k, delta, g, x_ref, y_ref, xs, s_ref, eta=eta, theta=theta, l1=l1)
    else:
        oracle.master_update_each(k, delta, g, x_ref, eta=eta, l1=l1)
    kx, dx, _ = oracle.quantize_wide(x_ref, bx, seed, it, oracle.MASTER_ID, oracle.TAG_MODEL)
    x, y, xsum = dev(x0), dev(y0), dev(sum0)
    nwx = dq.packed_words(d, bx)
    xq = torch.full((nwx + 4,), -1, dtype=torch.int32, device="cuda")
    dxo = torch.zeros(1, device="cuda")
    amx = torch.zeros(1, device="cuda")
    dq.dq_master_step_each(dev(pw.view(np.int32)), dev(delta), M, b, dev(g), x, y if acc else None, dev(xs),
                           xsum if acc else None, float(eta), float(theta), float(l1), bx, seed, it, xq, dxo, amx)
    assert np.array_equal(host(x).view(np.uint32), x_ref.view(np.uint32))
    if acc:
        assert np.array_equal(host(y).view(np.uint32), y_ref.view(np.uint32))
        assert np.array_equal(host(xsum).view(np.uint32), s_ref.view(np.uint32))
    assert host(dxo)[0] == dx and host(amx)[0] == oracle.absmax(x_ref)
    assert np.array_equal(words(xq)[:nwx], oracle.pack_wide(kx, bx))
    assert np.all(words(xq)[nwx:] == 0xFFFFFFFF)


def test_master_step_each_float_messages(dq):
    M, d = 5, 1003
    rng = np.random.default_rng(8)
    ld = 1004
    grads = np.zeros((M, ld), dtype=np.float32)
    grads[:, :d] = 0.1 * rng.standard_normal((M, d))
    g = (0.1 * rng.standard_normal(d)).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    x_ref = x0.copy()
    oracle.master_update_each_full(grads[:, :d], g, x_ref, eta=0.1, l1=0.01)
    x = dev(x0)
    xq = torch.zeros(d, dtype=torch.int32, device="cuda")
    one = torch.zeros(1, device="cuda")
    dq.dq_master_step_each(dev(grads.view(np.int32))[:, :d], None, M, 32, dev(g), x, None, None, None, 0.1, 0.0, 0.01, 32,
                           0, 0, xq, one, one.clone())
    assert np.array_equal(host(x).view(np.uint32), x_ref.view(np.uint32))
    assert np.array_equal(words(xq), x_ref.view(np.uint32))
