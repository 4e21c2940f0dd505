"""GPU parity on degenerate shapes: single coordinate, single row, empty CSR rows, batches far larger than a block's share."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle import algorithms as alg
from gpu_util import dev, host, words

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def dq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1805_10111_amd as dq
    return dq


def _dense_problem(dq, n, d, seed):
    p = synth.dense_logistic(n, d, seed=seed, l2=1e-3, l1=1e-4)
    lda = (d + 3) // 4 * 4
    Xp = np.zeros((n, lda), dtype=np.float32)
    Xp[:, :d] = p.dense
    return p, dq.DeviceProblem(n=n, d=d, y=dev(p.y), l2=p.l2, l1=p.l1, dense=dev(Xp)[:, :d])


def _check_worker(dq, p, P, M, B, b=8, sparsify=False):
    rp = oracle.RefProblem(p)
    d, n = p.d, p.n
    rng = np.random.default_rng(d + n)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    x = (x_snap + 0.05 * rng.standard_normal(d)).astype(np.float32)
    kx, dx, _ = oracle.quantize(x, 8, 3, 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    xq, q = oracle.pack(kx, 8), oracle.dequantize(kx, dx)
    seed, it = 21, 3
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    ld = (d + 3) // 4 * 4
    packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    alpha = torch.zeros((M, ld), device="cuda")[:, :d]
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    xq_d = torch.zeros(max(4, xq.size), dtype=torch.int32, device="cuda")
    xq_d[: xq.size] = dev(xq.view(np.int32))
    dq.dq_worker_step(P, None, M, B, xq_d, dev(np.array([dx], dtype=np.float32)), 8, False, dev(x_snap), None, sparsify,
                      b, seed, it, 0, packed, delta, None, alpha, None, ws)
    flips = 0
    for w in range(M):
        wd, dl, _, a_ref, _, _ = alg.worker_message(rp, q, x_snap, False, B, b, seed, it, w, sparsify)
        scale = max(np.abs(a_ref).max(), 1e-30)
        assert np.abs(host(alpha)[w].astype(np.float64) - a_ref).max() <= TOL * scale
        assert abs(host(delta)[w] - dl) <= 2e-5 * max(dl, 1e-30)
        k = oracle.unpack(words(packed)[w, :nw], d, b)
        flips += int(np.count_nonzero(k != oracle.unpack(wd, d, b)))
    assert flips <= max(3, 2e-3 * M * d)


@pytest.mark.parametrize("n,d,M,B", [(1, 1, 1, 1), (5, 3, 1, 1), (7, 2, 3, 9), (40, 260, 2, 700), (3, 1000, 2, 257)])
def test_dense_edge_shapes(dq, n, d, M, B):
    p, P = _dense_problem(dq, n, d, seed=n * 10 + d)
    rp = oracle.RefProblem(p)
    x = (0.5 * np.random.default_rng(1).standard_normal(d)).astype(np.float32)
    g = torch.zeros(d, device="cuda")
    z = torch.zeros(n, device="cuda")
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    xd = torch.zeros(max(4, d), device="cuda")[:d]
    xd.copy_(dev(x))
    dq.dq_full_grad(P, xd, g, z, obj, dq.new_workspace(dq.OP_FULL_GRAD, P))
    g_ref, z_ref = oracle.full_grad(rp, x, want_margins=True)
    assert np.abs(host(g) - g_ref).max() <= TOL * np.abs(g_ref).max()
    assert np.abs(host(z) - z_ref).max() <= TOL * max(np.abs(z_ref).max(), 1e-30)
    assert abs(host(obj)[0] - oracle.objective(rp, x)) <= TOL * oracle.objective(rp, x)
    _check_worker(dq, p, P, M, B)


def _csr(n, d, lens, seed):
    rng = np.random.default_rng(seed)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=indptr[1:])
    indices = np.concatenate([np.sort(rng.choice(d, size=l, replace=False)) for l in lens] + [np.zeros(0, dtype=np.int64)]).astype(np.int32)
    values = rng.standard_normal(int(indptr[-1])).astype(np.float32)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    return synth.Problem(n=n, d=d, y=y, l2=1e-3, l1=1e-4, indptr=indptr, indices=indices, values=values)


@pytest.mark.parametrize("case", ["one_row", "empty_rows", "all_empty", "one_column", "big_batch"])
def test_csr_edge_shapes(dq, case):
    if case == "one_row":
        p, M, B = _csr(1, 50, [7], 1), 2, 3
    elif case == "empty_rows":
        p, M, B = _csr(12, 40, [0, 3, 0, 0, 5, 1, 0, 2, 0, 4, 0, 6], 2), 3, 20
    elif case == "all_empty":
        p, M, B = _csr(6, 30, [0] * 6, 3), 2, 4
    elif case == "one_column":
        p, M, B = _csr(9, 1, [1, 0, 1, 1, 0, 1, 1, 1, 0], 4), 2, 5
    else:
        p, M, B = synth.sparse_text_logistic(300, 900, mean_nnz=12.0, seed=5), 2, 600
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    x = (0.5 * np.random.default_rng(1).standard_normal(p.d)).astype(np.float32)
    g = torch.zeros(p.d, device="cuda")
    z = torch.zeros(p.n, device="cuda")
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    xd = torch.zeros(max(4, p.d), device="cuda")[: p.d]
    xd.copy_(dev(x))
    dq.dq_full_grad(P, xd, g, z, obj, dq.new_workspace(dq.OP_FULL_GRAD, P))
    g_ref, z_ref = oracle.full_grad(rp, x, want_margins=True)
    assert np.abs(host(g) - g_ref).max() <= TOL * max(np.abs(g_ref).max(), 1e-30)
    assert np.abs(host(z) - z_ref).max() <= TOL * max(np.abs(z_ref).max(), 1e-30)
    assert abs(host(obj)[0] - oracle.objective(rp, x)) <= TOL * oracle.objective(rp, x)
    _check_worker(dq, p, P, M, B)
    _check_worker(dq, p, P, M, B, b=4, sparsify=True)
