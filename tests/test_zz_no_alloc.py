"""dq_worker_step_static (the worker step on the library's built-in workspace, for callers that cannot allocate)
against dq_worker_step, through the C ABI: identical messages bit for bit, on two calls in a row, the second one
on a smaller input, for dense and for CSR features."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import dev, host, words

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1805_10111_amd as dq
    return dq


def _model(rng, d, x_snap):
    x = (x_snap + 0.05 * rng.standard_normal(d)).astype(np.float32)
    k, dx, _ = oracle.quantize(x, 8, 3, 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    return oracle.pack(k, 8), dx


def _both(dq, P, M, B, xq, dx, x_snap, sparsify, b, seed, it):
    d = P.d
    nw = dq.packed_words(d, b)
    ldw, ld = (nw + 3) // 4 * 4, (d + 3) // 4 * 4
    outs = []
    for static in (True, False):
        packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
        delta = torch.zeros(M, device="cuda")
        nnz = torch.zeros(M, dtype=torch.int32, device="cuda")
        alpha = torch.zeros((M, ld), device="cuda")[:, :d]
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        args = (P, None, M, B, xq, dx, 8, False, x_snap, None, sparsify, b, seed, it, 0, packed, delta, nnz, alpha, status)
        if static:
            dq.dq_worker_step_static(*args)
        else:
            dq.dq_worker_step(*args, dq.new_workspace(dq.OP_VR_GRAD, P, M, B))
        torch.cuda.synchronize()
        outs.append((packed, delta, nnz, alpha, status))
    for a, b_ in zip(*outs):
        assert torch.equal(a, b_)
    assert outs[0][0][:, :nw].any() and host(outs[0][4])[0] == 0
    return outs[0]


def test_dense_two_calls_second_smaller(dq):
    n, d = 3000, 4096
    p = synth.dense_logistic(n, d, seed=21)
    P = dq.DeviceProblem.from_host(p)
    rng = np.random.default_rng(5)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx = _model(rng, d, x_snap)
    xq_d, dx_d, xs_d = dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), dev(x_snap)
    assert dq.dq_workspace_bytes(dq.OP_VR_GRAD, P, 32, 256) > 0          # partial sums do pass through a workspace
    packed, delta, _, alpha, _ = _both(dq, P, 32, 256, xq_d, dx_d, xs_d, False, 8, 11, 4)
    # the oracle's quantizer on the gradient of the built-in-workspace call: the same words
    for w in (0, 31):
        k, dl, _ = oracle.quantize(host(alpha)[w], 8, 11, 4, w)
        assert host(delta)[w] == dl and np.array_equal(words(packed)[w, :d // 4], oracle.pack(k, 8))
    _both(dq, P, 8, 64, xq_d, dx_d, xs_d, False, 4, 11, 5)               # smaller: fewer workers, smaller batches
    # a narrower problem after the wide one
    p2 = synth.dense_logistic(500, 1500, seed=22)
    P2 = dq.DeviceProblem.from_host(p2)
    xs2 = (0.3 * rng.standard_normal(1500)).astype(np.float32)
    xq2, dx2 = _model(rng, 1500, xs2)
    _both(dq, P2, 5, 48, dev(xq2.view(np.int32)), dev(np.array([dx2], dtype=np.float32)), dev(xs2), True, 4, 11, 6)


def test_csr_two_calls_second_smaller(dq):
    cfg = synth.CONFIGS["C3"]
    p = synth.make_problem(cfg, n=6000)
    P = dq.DeviceProblem.from_host(p)
    d = p.d
    rng = np.random.default_rng(6)
    x_snap = (0.05 * rng.standard_normal(d)).astype(np.float32)
    xq, dx = _model(rng, d, x_snap)
    xq_d, dx_d, xs_d = dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), dev(x_snap)
    _both(dq, P, 16, 64, xq_d, dx_d, xs_d, True, 4, 9, 2)                # Alg. 2: the sparsified gradient crosses the workspace
    _both(dq, P, 4, 16, xq_d, dx_d, xs_d, True, 4, 9, 3)
    _both(dq, P, 8, 32, xq_d, dx_d, xs_d, False, 8, 9, 4)
    # many workers: a single step still fits, although the workspace of a run (which also holds what dq_run_rounds
    # keeps between rounds) would not
    assert dq.dq_workspace_bytes(dq.OP_WORKER_STEP, P, 64, 8) <= dq.STATIC_WS_BYTES < dq.dq_workspace_bytes(dq.OP_VR_GRAD, P, 64, 8)
    _both(dq, P, 64, 8, xq_d, dx_d, xs_d, True, 4, 9, 5)


def test_too_large_for_the_builtin_workspace(dq):
    p = synth.dense_logistic(64, 16384, seed=1)
    P = dq.DeviceProblem.from_host(p)
    d, M, B = 16384, 64, 256
    assert dq.dq_workspace_bytes(dq.OP_WORKER_STEP, P, M, B) > dq.STATIC_WS_BYTES
    z = torch.zeros(d, device="cuda")
    packed = torch.zeros((M, d // 4), dtype=torch.int32, device="cuda")
    with pytest.raises(dq.DqError) as e:
        dq.dq_worker_step_static(P, None, M, B, packed[0], z[:1], 8, False, z, None, False, 8, 0, 0, 0, packed,
                                 torch.zeros(M, device="cuda"))
    assert e.value.code == dq.ERR_WORKSPACE
