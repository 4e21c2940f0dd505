"""GPU parity: dense full gradient, variance-reduced gradient and fused worker step versus the oracle.

Floating-point results are compared at 1e-5 relative to the largest entry of the oracle's
vector (the oracle accumulates in double, the kernels in float32).  Integer results (codes)
are compared bit-exactly against the library's own unfused chain, and against the oracle
up to the rounding decisions that a sub-tolerance difference of alpha can flip.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import dev, host, words

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def dq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1805_10111_amd as dq
    return dq


def _ws(dq, op, P, M=1, B=1):
    return dq.new_workspace(op, P, M, B)


def _close(got, want, tol=TOL):
    scale = np.abs(want).max()
    assert np.abs(got.astype(np.float64) - want).max() <= tol * scale + 1e-30, \
        (np.abs(got.astype(np.float64) - want).max(), scale)


def _model(rng, d, b_x, x_snap, spread=0.05):
    """A model near the snapshot and its b_x-bit message (packed words, delta, dequantized q) from the oracle."""
    x = (x_snap + spread * rng.standard_normal(d)).astype(np.float32)
    if b_x == 32:
        return x.view(np.uint32).copy(), np.float32(1.0), x
    k, dx, _ = oracle.quantize(x, b_x, 3, 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    return oracle.pack(k, b_x), dx, oracle.dequantize(k, dx)


# (the last two give a block more rows than one chunk of labels/margins holds: 1024, then a ragged remainder)
PROBLEMS = [(2000, 1000), (37, 13), (300, 4096), (129, 2048), (64, 1027), (150, 6000), (90, 16384), (70, 12003),
            (600011, 8), (1100000, 5)]


@pytest.mark.parametrize("n,d", PROBLEMS)
def test_full_grad(dq, n, d):
    p = synth.dense_logistic(n, d, seed=n + d, l2=1e-3, l1=1e-4)
    lda = (d + 3) // 4 * 4
    if lda != d:                                   # padded rows: padding must be ignored
        Xp = np.full((n, lda), 7.0, dtype=np.float32)
        Xp[:, :d] = p.dense
    else:
        Xp = p.dense
    P = dq.DeviceProblem(n=n, d=d, y=dev(p.y), l2=p.l2, l1=p.l1, dense=dev(Xp)[:, :d])
    rp = oracle.RefProblem(p)
    x = (0.5 * np.random.default_rng(1).standard_normal(d)).astype(np.float32)
    g = torch.zeros(d, device="cuda")
    z = torch.zeros(n, device="cuda")
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = _ws(dq, dq.OP_FULL_GRAD, P)
    dq.dq_full_grad(P, dev(x), g, z, obj, ws)
    g_ref, z_ref = oracle.full_grad(rp, x, want_margins=True)
    _close(host(g), g_ref.astype(np.float64))
    _close(host(z), z_ref.astype(np.float64))
    assert abs(host(obj)[0] - oracle.objective(rp, x)) <= TOL * oracle.objective(rp, x)
    # deterministic: a second call gives the same bits
    g2 = torch.zeros(d, device="cuda")
    dq.dq_full_grad(P, dev(x), g2, None, None, ws)
    assert torch.equal(g, g2)


@pytest.mark.parametrize("have_z", [True, False])
@pytest.mark.parametrize("b_x", [8, 4, 32])
@pytest.mark.parametrize("n,d,M,B", [(2000, 1000, 4, 16), (300, 4096, 3, 40), (64, 1027, 2, 5), (500, 2048, 33, 7),
                                     (150, 6000, 3, 40), (90, 16384, 2, 9), (70, 12003, 2, 33)])
def test_vr_grad(dq, n, d, M, B, b_x, have_z):
    p = synth.dense_logistic(n, d, seed=d, l2=1e-3)
    P = dq.DeviceProblem.from_host(p) if d % 4 == 0 else None
    if P is None:
        lda = (d + 3) // 4 * 4
        Xp = np.zeros((n, lda), dtype=np.float32)
        Xp[:, :d] = p.dense
        P = dq.DeviceProblem(n=n, d=d, y=dev(p.y), l2=p.l2, l1=p.l1, dense=dev(Xp)[:, :d])
    rp = oracle.RefProblem(p)
    rng = np.random.default_rng(5)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, q = _model(rng, d, b_x, x_snap)
    idx = np.stack([oracle.sample_indices(n, B, 11, 2, w) for w in range(M)])
    z_snap = None
    if have_z:
        _, z_ref = oracle.full_grad(rp, x_snap, want_margins=True)
        z_snap = dev(z_ref)
    ld = (d + 3) // 4 * 4
    alpha = torch.full((M, ld), 5.0, device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    l1n = torch.zeros(M, device="cuda")
    ws = _ws(dq, dq.OP_VR_GRAD, P, M, B)
    dq.dq_vr_grad(P, dev(idx), M, B, dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), b_x, False,
                  dev(x_snap), z_snap, alpha, amax, l1n, ws)
    for w in range(M):
        want = oracle.vr_grad(rp, idx[w], q, x_snap).astype(np.float64)
        got = host(alpha)[w]
        _close(got, want)
        assert host(amax)[w] == np.abs(got).max()
        assert abs(host(l1n)[w] - np.abs(got.astype(np.float64)).sum()) <= 1e-6 * np.abs(got).sum()


def test_vr_grad_flag_bit_and_bad_index(dq):
    n, d, M, B = 200, 1000, 3, 8
    p = synth.dense_logistic(n, d, seed=2)
    P = dq.DeviceProblem.from_host(p)
    x_snap = dev(np.random.default_rng(0).standard_normal(d).astype(np.float32))
    idx = torch.zeros((M, B), dtype=torch.int32, device="cuda")
    alpha = torch.full((M, d), 5.0, device="cuda")
    amax = torch.full((M,), 5.0, device="cuda")
    ws = _ws(dq, dq.OP_VR_GRAD, P, M, B)
    dq.dq_vr_grad(P, idx, M, B, None, None, 8, True, x_snap, None, alpha, amax, None, ws)
    assert not host(alpha).any() and not host(amax).any()
    # worker step in the flag-bit round: zero codes, delta = 0
    packed = torch.full((M, 252), -1, dtype=torch.int32, device="cuda")
    delta = torch.full((M,), 5.0, device="cuda")
    nnz = torch.full((M,), 5, dtype=torch.int32, device="cuda")
    dq.dq_worker_step(P, idx, M, B, None, None, 8, True, x_snap, None, False, 8, 1, 1, 0, packed, delta, nnz, None, None, ws)
    assert not words(packed)[:, :250].any() and not host(delta).any() and not host(nnz).any()
    # indices outside [0, n) are skipped, not dereferenced
    bad = torch.tensor([[0, -1, n, 2 ** 31 - 1, 1, 2, 3, 4]] * M, dtype=torch.int32, device="cuda")
    xq = torch.zeros(250, dtype=torch.int32, device="cuda")
    dq.dq_vr_grad(P, bad, M, B, xq, torch.ones(1, device="cuda"), 8, False, x_snap, None, alpha, amax, None, ws)
    assert np.isfinite(host(alpha)).all()


@pytest.mark.parametrize("bad", [False, True])
@pytest.mark.parametrize("d,M,B", [(4096, 2, 256), (4096, 1, 71), (3000, 2, 70), (4096, 32, 64), (2052, 3, 44),
                                   (2048, 2, 70), (1500, 3, 64), (8192, 2, 40), (6000, 2, 70), (16384, 2, 36),
                                   (12000, 1, 33), (4096, 1, 65536), (2048, 1, 40000),
                                   (1024, 3, 64), (1028, 2, 40), (4100, 2, 40), (8196, 2, 36), (16380, 1, 34)])
def test_vr_grad_row_streaming_paths(dq, d, M, B, bad):
    """Rows wider than 1024 floats are streamed with two row buffers when a block owns whole pairs of batches of valid
    rows, with one buffer when it owns whole batches, and through the checked loop otherwise (ragged last block,
    indices outside [0, n)).  Every path against the oracle; a skipped index contributes nothing but still counts
    in the 1/B of the mean."""
    n = 400
    p = synth.dense_logistic(n, d, seed=d + B, l2=1e-3)
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    rng = np.random.default_rng(B)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, q = _model(rng, d, 8, x_snap)
    idx = np.stack([oracle.sample_indices(n, B, 17, 3, w) for w in range(M)]).astype(np.int64)
    if bad:                                              # a few rows of every worker are out of range
        for w in range(M):
            pos = rng.choice(B, size=max(1, B // 9), replace=False)
            idx[w, pos] = rng.choice([-1, n, n + 5, 2 ** 31 - 1], size=pos.size)
    _, z_ref = oracle.full_grad(rp, x_snap, want_margins=True)
    alpha = torch.full((M, d), 5.0, device="cuda")
    amax = torch.zeros(M, device="cuda")
    ws = _ws(dq, dq.OP_VR_GRAD, P, M, B)
    dq.dq_vr_grad(P, dev(idx.astype(np.int32)), M, B, dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), 8, False,
                  dev(x_snap), dev(z_ref), alpha, amax, None, ws)
    dense_part = p.l2 * (q.astype(np.float64) - x_snap.astype(np.float64))
    for w in range(M):
        ok = idx[w][(idx[w] >= 0) & (idx[w] < n)]
        want = (oracle.vr_grad(rp, ok.astype(np.int32), q, x_snap).astype(np.float64) - dense_part) * (ok.size / B) + dense_part
        _close(host(alpha)[w], want, tol=2e-5 if bad else TOL)   # (the oracle's float32 output is rescaled here)
        assert host(amax)[w] == np.abs(host(alpha)[w]).max()


@pytest.mark.parametrize("sparsify", [False, True])
@pytest.mark.parametrize("b", [8, 4, 2])
@pytest.mark.parametrize("n,d,M,B", [(2000, 1000, 4, 16), (300, 4096, 5, 64), (64, 1027, 2, 5), (150, 6000, 3, 40),
                                     (90, 16384, 2, 9)])
def test_worker_step(dq, n, d, M, B, b, sparsify):
    p = synth.dense_logistic(n, d, seed=d + 1, l2=1e-3)
    lda = (d + 3) // 4 * 4
    Xp = np.zeros((n, lda), dtype=np.float32)
    Xp[:, :d] = p.dense
    P = dq.DeviceProblem(n=n, d=d, y=dev(p.y), l2=p.l2, l1=p.l1, dense=dev(Xp)[:, :d])
    rp = oracle.RefProblem(p)
    rng = np.random.default_rng(6)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, q = _model(rng, d, 8, x_snap)
    seed, it, w0 = 77, 9, 100
    idx = np.stack([oracle.sample_indices(n, B, seed, it, w0 + w) for w in range(M)])
    xs_d, xq_d, dx_d, idx_d = dev(x_snap), dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), dev(idx)
    ws = _ws(dq, dq.OP_VR_GRAD, P, M, B)
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    # fused
    packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    nnz = torch.zeros(M, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    alpha_f = torch.zeros((M, lda), device="cuda")[:, :d]
    dq.dq_worker_step(P, idx_d, M, B, xq_d, dx_d, 8, False, xs_d, None, sparsify, b, seed, it, w0, packed, delta, nnz,
                      alpha_f, status, ws)
    # unfused chain of the same library: must agree bit for bit
    alpha = torch.zeros((M, lda), device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    dq.dq_vr_grad(P, idx_d, M, B, xq_d, dx_d, 8, False, xs_d, None, alpha, amax, None, ws)
    assert torch.equal(alpha, alpha_f)
    v = alpha
    if sparsify:
        beta = torch.zeros((M, lda), device="cuda")[:, :d]
        kept = torch.zeros(M, dtype=torch.int32, device="cuda")
        dq.dq_sparsify(alpha, None, seed, it, w0, beta, amax, kept)
        v = beta
    packed2 = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    delta2 = torch.zeros(M, device="cuda")
    dq.dq_quantize_pack(v, b, amax, True, seed, it, dq.TAG_GRAD, w0, packed2, delta2)
    assert torch.equal(packed[:, :nw], packed2[:, :nw]) and torch.equal(delta, delta2)
    assert np.all(words(packed)[:, nw:] == 0xFFFFFFFF)
    assert host(status)[0] == 0
    # against the oracle: the decoded message is an unbiased rounding of the oracle's vector
    flips = 0
    for w in range(M):
        a_ref = oracle.vr_grad(rp, idx[w], q, x_snap)
        _close(host(alpha_f)[w], a_ref.astype(np.float64))
        v_ref = oracle.sparsify(a_ref, seed, it, w0 + w)[0] if sparsify else a_ref
        k_ref, d_ref, _ = oracle.quantize(v_ref, b, seed, it, w0 + w)
        k = oracle.unpack(words(packed)[w, :nw], d, b)
        assert host(nnz)[w] == np.count_nonzero(k)
        assert abs(host(delta)[w] - d_ref) <= 2e-5 * d_ref
        diff = np.abs(k.astype(np.int32) - k_ref.astype(np.int32))
        if not sparsify:
            assert diff.max() <= 1
            flips += int(diff.sum())
        else:
            # a flipped keep decision changes a code by the full level; count them
            flips += int(np.count_nonzero(diff))
    assert flips <= max(3, 2e-3 * M * d), flips          # decisions flipped by sub-tolerance differences
    # the direct check: the oracle's sparsifier and quantizer applied to the gradient the GPU itself computed give
    # the GPU's message word for word (identical quantizer inputs => identical codes, no flips)
    for w in range(M):
        a_gpu = host(alpha_f)[w]
        v_o = oracle.sparsify(a_gpu, seed, it, w0 + w)[0] if sparsify else a_gpu
        k_o, d_o, _ = oracle.quantize(v_o, b, seed, it, w0 + w)
        assert host(delta)[w] == d_o
        assert np.array_equal(words(packed)[w, :nw], oracle.pack(k_o, b))
        assert host(nnz)[w] == np.count_nonzero(k_o)


def test_worker_step_samples_its_own_minibatch(dq):
    """idx = None: the kernel draws the mini-batch itself, identically to dq_sample_indices."""
    n, d, M, B = 2000, 1000, 4, 16
    p = synth.dense_logistic(n, d, seed=8)
    P = dq.DeviceProblem.from_host(p)
    rng = np.random.default_rng(2)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, _ = _model(rng, d, 8, x_snap)
    seed, it, w0 = 5, 17, 3
    idx = torch.zeros((M, B), dtype=torch.int32, device="cuda")
    dq.dq_sample_indices(n, M, B, seed, it, w0, idx)
    ws = _ws(dq, dq.OP_VR_GRAD, P, M, B)
    outs = []
    for use_idx in (idx, None):
        packed = torch.zeros((M, 252), dtype=torch.int32, device="cuda")
        delta = torch.zeros(M, device="cuda")
        dq.dq_worker_step(P, use_idx, M, B, dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), 8, False,
                          dev(x_snap), None, False, 8, seed, it, w0, packed, delta, None, None, None, ws)
        outs.append((packed, delta))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert outs[0][0].any()


def test_worker_step_full_precision_message(dq):
    """b = 32: the worker sends alpha itself (AsyFPG / QSVRG-style comparison modes)."""
    n, d, M, B = 300, 1000, 2, 8
    p = synth.dense_logistic(n, d, seed=3)
    P = dq.DeviceProblem.from_host(p)
    rng = np.random.default_rng(1)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    x = (x_snap + 0.05 * rng.standard_normal(d)).astype(np.float32)
    idx = dev(np.stack([oracle.sample_indices(n, B, 1, 1, w) for w in range(M)]))
    ws = _ws(dq, dq.OP_VR_GRAD, P, M, B)
    out = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    alpha = torch.zeros((M, d), device="cuda")
    dq.dq_worker_step(P, idx, M, B, dev(x).view(torch.int32), None, 32, False, dev(x_snap), None, False, 32, 1, 1, 0,
                      out.view(torch.int32), delta, None, alpha, None, ws)
    assert torch.equal(out, alpha) and host(delta).tolist() == [1.0, 1.0]
    rp = oracle.RefProblem(p)
    for w in range(M):
        _close(host(out)[w], oracle.vr_grad(rp, host(idx)[w], x, x_snap).astype(np.float64))


def test_unsupported_and_invalid(dq):
    p = synth.dense_logistic(20, 16388, seed=0)
    P = dq.DeviceProblem.from_host(p)
    x = torch.zeros(16388, device="cuda")
    with pytest.raises(dq.DqError) as e:
        dq.dq_full_grad(P, x, x.clone(), None, None, torch.zeros(1 << 20, device="cuda"))
    assert e.value.code == dq.ERR_UNSUPPORTED             # dense rows wider than 16384 floats have no kernel
    p = synth.dense_logistic(20, 64, seed=0)
    P = dq.DeviceProblem.from_host(p)
    x = torch.zeros(64, device="cuda")
    with pytest.raises(dq.DqError) as e:
        dq.dq_full_grad(P, x, x.clone(), None, None, torch.zeros(4, device="cuda"))
    assert e.value.code == dq.ERR_WORKSPACE
