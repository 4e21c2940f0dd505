"""GPU parity at the full sizes of the configs, in the launch shapes the benchmark uses.

The oracle checks what it can reach in seconds: the whole full gradient, the gradients of a
few sampled workers, and one whole master step fed with the oracle's own messages.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import algorithms as alg
import synth
from gpu_util import dev, host, words

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def dq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1805_10111_amd as dq
    return dq


def _close(got, want, tol=TOL):
    scale = np.abs(want).max()
    err = np.abs(got.astype(np.float64) - want).max()
    assert err <= tol * scale + 1e-30, (err, scale)


@pytest.mark.parametrize("name", ["C4", "C2", "C3"])
def test_one_round_at_full_size(dq, name):
    cfg = synth.CONFIGS[name]
    p = synth.make_problem(cfg)
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    d, n, M, B, b, bx = p.d, p.n, cfg.M, cfg.B, cfg.b, cfg.b_x
    sparse = cfg.algo == "sparse"
    rng = np.random.default_rng(1)
    x_snap = (0.05 * rng.standard_normal(d)).astype(np.float32)
    x = (x_snap + 0.01 * rng.standard_normal(d)).astype(np.float32)
    seed, it = 5, 40
    # ---- epoch prologue: whole vectors
    g = torch.zeros(d, device="cuda")
    z = torch.zeros(n, device="cuda")
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    dq.dq_full_grad(P, dev(x_snap), g, z, obj, dq.new_workspace(dq.OP_FULL_GRAD, P))
    g_ref, z_ref = oracle.full_grad(rp, x_snap, want_margins=True)
    _close(host(g), g_ref.astype(np.float64))
    _close(host(z), z_ref.astype(np.float64))
    assert abs(host(obj)[0] - oracle.objective(rp, x_snap)) <= TOL * oracle.objective(rp, x_snap)
    # ---- master (i): the model message, bit-exact
    kx, dx, _ = oracle.quantize(x, bx, seed, it, oracle.MASTER_ID, oracle.TAG_MODEL)
    xq_ref = oracle.pack(kx, bx)
    q = oracle.dequantize(kx, dx)
    xq = torch.zeros(dq.packed_words(d, bx), dtype=torch.int32, device="cuda")
    dxo, amx = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
    dq.dq_quantize_pack(dev(x), bx, amx, False, seed, it, dq.TAG_MODEL, dq.MASTER_ID, xq, dxo)
    assert np.array_equal(words(xq), xq_ref) and host(dxo)[0] == dx
    # ---- worker side of the round, all M workers in one call, cached margins, in-kernel sampling
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    packed = torch.zeros((M, ldw), dtype=torch.int32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    nnz = torch.zeros(M, dtype=torch.int32, device="cuda")
    alpha = torch.zeros((M, (d + 3) // 4 * 4), device="cuda")[:, :d]
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    dq.dq_worker_step(P, None, M, B, xq, dxo, bx, False, dev(x_snap), z, sparse, b, seed, it, 0, packed, delta, nnz,
                      alpha, status, ws)
    assert host(status)[0] == 0
    flips = 0
    for w in (0, M // 2, M - 1):
        wd, dl, _, a_ref, _, _ = alg.worker_message(rp, q, x_snap, False, B, b, seed, it, w, sparse)
        _close(host(alpha)[w], a_ref.astype(np.float64))
        k = oracle.unpack(words(packed)[w, :nw], d, b)
        k_ref = oracle.unpack(wd, d, b)
        assert abs(host(delta)[w] - dl) <= 2e-5 * dl
        assert host(nnz)[w] == np.count_nonzero(k)
        flips += int(np.count_nonzero(k != k_ref))
    assert flips <= max(3, 2e-3 * 3 * d), flips
    # the direct check, every worker: the oracle's sparsifier and quantizer applied to the gradient the GPU itself
    # computed give the GPU's message word for word
    for w in range(M):
        a_gpu = host(alpha)[w]
        v_o = oracle.sparsify(a_gpu, seed, it, w)[0] if sparse else a_gpu
        k_o, d_o, _ = oracle.quantize(v_o, b, seed, it, w)
        assert host(delta)[w] == d_o
        assert np.array_equal(words(packed)[w, :nw], oracle.pack(k_o, b))
        assert host(nnz)[w] == np.count_nonzero(k_o)
    # ---- master (ii)+(i) at full M, fed with the oracle's messages: bit-exact
    codes = np.zeros((M, d), dtype=np.int8)
    deltas = np.zeros(M, dtype=np.float32)
    pw = np.zeros((M, ldw), dtype=np.uint32)
    for w in range(M):
        wd, dl, *_ = alg.worker_message(rp, q, x_snap, False, B, b, seed, it, w, sparse)
        pw[w, :nw] = wd
        codes[w] = oracle.unpack(wd, d, b)
        deltas[w] = dl
    y0 = (x + 0.01 * rng.standard_normal(d)).astype(np.float32)
    s0 = rng.standard_normal(d).astype(np.float32)
    acc = cfg.algo == "acc"
    eta, theta = np.float32(0.3), np.float32(0.5)
    x_ref, y_ref, s_ref = x.copy(), y0.copy(), s0.copy()
    if acc:
        oracle.master_update(codes, deltas, np.float32(1 / M), g_ref, x_ref, y_ref, x_snap, s_ref, eta=eta, theta=theta, l1=rp.l1)
    else:
        oracle.master_update(codes, deltas, np.float32(1 / M), g_ref, x_ref, eta=eta, l1=rp.l1)
    kx2, dx2, _ = oracle.quantize(x_ref, bx, seed, it + 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    xd, yd, sd = dev(x), dev(y0), dev(s0)
    dq.dq_master_step(dev(pw.view(np.int32)), dev(deltas), M, b, float(np.float32(1 / M)), dev(g_ref), xd,
                      yd if acc else None, dev(x_snap), sd if acc else None, float(eta), float(theta), float(rp.l1),
                      bx, seed, it + 1, xq, dxo, amx)
    assert np.array_equal(host(xd).view(np.uint32), x_ref.view(np.uint32))
    if acc:
        assert np.array_equal(host(yd), y_ref) and np.array_equal(host(sd), s_ref)
    assert np.array_equal(words(xq), oracle.pack(kx2, bx)) and host(dxo)[0] == dx2


def test_full_size_model_width_11_and_per_gradient_master(dq):
    """C2 at full size with a model message whose fields straddle words (b_x = 11) and the master applying
    every gradient as its own update."""
    cfg = synth.CONFIGS["C2"]
    p = synth.make_problem(cfg)
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    d, n, M, B, b, bx = p.d, p.n, cfg.M, cfg.B, cfg.b, 11
    rng = np.random.default_rng(2)
    x_snap = (0.05 * rng.standard_normal(d)).astype(np.float32)
    x = (x_snap + 0.01 * rng.standard_normal(d)).astype(np.float32)
    seed, it = 9, 17
    kx, dx, _ = oracle.quantize_wide(x, bx, seed, it, oracle.MASTER_ID, oracle.TAG_MODEL)
    q = oracle.dequantize_wide(kx, dx)
    xq = torch.zeros(dq.packed_words(d, bx), dtype=torch.int32, device="cuda")
    dxo, amx = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
    dq.dq_quantize_pack(dev(x), bx, amx, False, seed, it, dq.TAG_MODEL, dq.MASTER_ID, xq, dxo)
    assert np.array_equal(words(xq), oracle.pack_wide(kx, bx)) and host(dxo)[0] == dx
    # worker side on the 11-bit model
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    packed = torch.zeros((M, ldw), dtype=torch.int32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    alpha = torch.zeros((M, (d + 3) // 4 * 4), device="cuda")[:, :d]
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    dq.dq_worker_step(P, None, M, B, xq, dxo, bx, False, dev(x_snap), None, False, b, seed, it, 0, packed, delta, None,
                      alpha, None, ws)
    pw = np.zeros((M, ldw), dtype=np.uint32)
    codes = np.zeros((M, d), dtype=np.int8)
    deltas = np.zeros(M, dtype=np.float32)
    for w in range(M):
        wd, dl, _, a_ref, _, _ = alg.worker_message(rp, q, x_snap, False, B, b, seed, it, w, False)
        if w in (0, M - 1):
            _close(host(alpha)[w], a_ref.astype(np.float64))
        pw[w, :nw], codes[w], deltas[w] = wd, oracle.unpack(wd, d, b), dl
    # master: one update per gradient, new model again at 11 bits, fed with the oracle's messages: bit-exact
    g_ref = oracle.full_grad(rp, x_snap)
    eta = np.float32(0.05)
    x_ref = x.copy()
    oracle.master_update_each(codes, deltas, g_ref, x_ref, eta=eta, l1=rp.l1)
    kx2, dx2, _ = oracle.quantize_wide(x_ref, bx, seed, it + 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    xd = dev(x)
    dq.dq_master_step_each(dev(pw.view(np.int32)), dev(deltas), M, b, dev(g_ref), xd, None, None, None, float(eta), 0.0,
                           float(rp.l1), bx, seed, it + 1, xq, dxo, amx)
    assert np.array_equal(host(xd).view(np.uint32), x_ref.view(np.uint32))
    assert np.array_equal(words(xq), oracle.pack_wide(kx2, bx)) and host(dxo)[0] == dx2


def test_dense_matrix_beyond_2_to_31_elements(dq):
    """A dense matrix of 655,360 x 4096 floats (10.7 GB): element offsets pass 2^31 and byte offsets 2^33.  The
    device matrix is a seeded block of 8192 rows repeated 80 times, so the oracle can work on the block: row i
    of the matrix is row i mod 8192 of the block, and the mean over all rows equals the mean over the block."""
    nb, reps, d = 8192, 80, 4096
    p = synth.dense_logistic(nb, d, seed=3, l2=1e-4)
    rp = oracle.RefProblem(p)
    n = nb * reps
    X = dev(p.dense).repeat(reps, 1)
    assert X.numel() > 2 ** 31 and X.is_contiguous()
    P = dq.DeviceProblem(n=n, d=d, y=dev(p.y).repeat(reps), l2=p.l2, l1=p.l1, dense=X)
    rng = np.random.default_rng(4)
    x_snap = (0.05 * rng.standard_normal(d)).astype(np.float32)
    # ---- whole gradient and margins
    g = torch.zeros(d, device="cuda")
    z = torch.zeros(n, device="cuda")
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    dq.dq_full_grad(P, dev(x_snap), g, z, obj, dq.new_workspace(dq.OP_FULL_GRAD, P))
    g_ref, z_ref = oracle.full_grad(rp, x_snap, want_margins=True)
    _close(host(g), g_ref.astype(np.float64))
    zh = host(z).reshape(reps, nb)
    _close(zh[0], z_ref.astype(np.float64))
    assert all(np.array_equal(zh[r], zh[0]) for r in range(1, reps))
    assert abs(host(obj)[0] - oracle.objective(rp, x_snap)) <= TOL * oracle.objective(rp, x_snap)
    # ---- worker gradients from rows in the last 8192 (offsets of 2.6e9 elements and more), given and drawn
    M, B, bx = 8, 64, 8
    x = (x_snap + 0.01 * rng.standard_normal(d)).astype(np.float32)
    kx, dx, _ = oracle.quantize(x, bx, 5, 0, oracle.MASTER_ID, oracle.TAG_MODEL)
    q = oracle.dequantize(kx, dx)
    xq = dev(oracle.pack(kx, bx).view(np.int32))
    idx_small = rng.integers(0, nb, size=(M, B))
    idx = idx_small + (n - nb)
    alpha = torch.zeros((M, d), device="cuda")
    amax = torch.zeros(M, device="cuda")
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    dq.dq_vr_grad(P, dev(idx.astype(np.int32)), M, B, xq, dev(np.array([dx], dtype=np.float32)), bx, False, dev(x_snap), z,
                  alpha, amax, None, ws)
    for w in range(M):
        _close(host(alpha)[w], oracle.vr_grad(rp, idx_small[w].astype(np.int32), q, x_snap).astype(np.float64))
    # rows drawn in the kernel (worker step): uniform on [0, n), four in five past element 2^31 / 4
    b, nw = 8, dq.packed_words(d, 8)
    packed = torch.zeros((M, nw), dtype=torch.int32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    dq.dq_worker_step(P, None, M, B, xq, dev(np.array([dx], dtype=np.float32)), bx, False, dev(x_snap), z, False, b, 11, 2, 0,
                      packed, delta, None, alpha, status, ws)
    assert host(status)[0] == 0
    for w in (0, M - 1):
        drawn = oracle.sample_indices(n, B, 11, 2, w)
        assert drawn.max() >= nb * (reps // 2)
        a_ref = oracle.vr_grad(rp, (drawn % nb).astype(np.int32), q, x_snap)
        _close(host(alpha)[w], a_ref.astype(np.float64))
        assert abs(host(delta)[w] - np.abs(a_ref).max() / 127) <= 2e-5 * host(delta)[w]


def test_csr_matrix_beyond_2_to_31_entries(dq):
    """A CSR matrix with 2.2e9 stored entries (entry offsets pass 2^31): a seeded block of 12,000 rows repeated 3500
    times on the device; the oracle works on the block (row i of the matrix is row i mod 12,000 of the block)."""
    nb, reps, d = 12000, 3500, 20958
    p = synth.sparse_text_logistic(nb, d, mean_nnz=52.0, seed=8)
    rp = oracle.RefProblem(p)
    nnz_b = int(p.indptr[-1])
    n = nb * reps
    assert nnz_b * reps > 2 ** 31
    shifts = torch.arange(reps, device="cuda", dtype=torch.int64) * nnz_b
    indptr = torch.cat([(dev(p.indptr[:-1])[None, :] + shifts[:, None]).reshape(-1),
                        torch.tensor([nnz_b * reps], device="cuda", dtype=torch.int64)])
    P = dq.DeviceProblem(n=n, d=d, y=dev(p.y).repeat(reps), l2=p.l2, l1=p.l1, indptr=indptr,
                         indices=dev(p.indices).repeat(reps), values=dev(p.values).repeat(reps))
    rng = np.random.default_rng(4)
    x_snap = (0.05 * rng.standard_normal(d)).astype(np.float32)
    g = torch.zeros(d, device="cuda")
    z = torch.zeros(n, device="cuda")
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    dq.dq_full_grad(P, dev(x_snap), g, z, obj, dq.new_workspace(dq.OP_FULL_GRAD, P))
    g_ref, z_ref = oracle.full_grad(rp, x_snap, want_margins=True)
    _close(host(g), g_ref.astype(np.float64))
    zh = host(z).reshape(reps, nb)
    _close(zh[0], z_ref.astype(np.float64))
    assert np.array_equal(zh[-1], zh[0]) and np.array_equal(zh[reps // 2], zh[0])
    assert abs(host(obj)[0] - oracle.objective(rp, x_snap)) <= TOL * oracle.objective(rp, x_snap)
    # ---- worker gradients from rows of the last block (entry offsets of 2.2e9)
    M, B, bx = 8, 32, 8
    x = (x_snap + 0.01 * rng.standard_normal(d)).astype(np.float32)
    kx, dx, _ = oracle.quantize(x, bx, 5, 0, oracle.MASTER_ID, oracle.TAG_MODEL)
    q = oracle.dequantize(kx, dx)
    xq = dev(oracle.pack(kx, bx).view(np.int32))
    idx_small = rng.integers(0, nb, size=(M, B))
    idx = idx_small + (n - nb)
    alpha = torch.zeros((M, (d + 3) // 4 * 4), device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    dq.dq_vr_grad(P, dev(idx.astype(np.int32)), M, B, xq, dev(np.array([dx], dtype=np.float32)), bx, False, dev(x_snap), z,
                  alpha, amax, None, ws)
    for w in range(M):
        _close(host(alpha)[w], oracle.vr_grad(rp, idx_small[w].astype(np.int32), q, x_snap).astype(np.float64))
