"""GPU parity: CSR full gradient, variance-reduced gradient and fused worker step versus the oracle."""
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


def _close(got, want, tol=TOL):
    scale = np.abs(want).max()
    err = np.abs(got.astype(np.float64) - want).max()
    assert err <= tol * scale + 1e-30, (err, scale)


def _long_rows_problem(n=40, d=20958, seed=0):
    """CSR with a few very long rows: exercises staging groups and the unstaged path."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, 80, size=n)
    lens[3] = 10000
    lens[7] = lens[8] = lens[9] = 3000
    lens[20] = 1
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=indptr[1:])
    indices = np.concatenate([np.sort(rng.choice(d, size=l, replace=False)) for l in lens]).astype(np.int32)
    values = (rng.standard_normal(indptr[-1]) / np.sqrt(np.repeat(lens, lens))).astype(np.float32)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    return synth.Problem(n=n, d=d, y=y, l2=1e-3, l1=1e-4, indptr=indptr, indices=indices, values=values)


def _widest_problem():
    """2^20 - 1 columns, and the last column (the largest index a staged entry can carry) present in several rows."""
    p = synth.sparse_text_logistic(300, (1 << 20) - 1, mean_nnz=40.0, seed=5)
    indices = p.indices.copy()
    for r in range(0, 300, 7):
        if p.indptr[r + 1] > p.indptr[r]:
            indices[p.indptr[r + 1] - 1] = p.d - 1          # rows stay sorted: the last entry gets the last column
    return synth.Problem(n=p.n, d=p.d, y=p.y, l2=p.l2, l1=p.l1, indptr=p.indptr, indices=indices, values=p.values)


def _problems():
    return {
        "text": synth.sparse_text_logistic(3000, 20958, seed=1),
        "tiny": synth.sparse_text_logistic(60, 50, mean_nnz=6.0, seed=2, l2=1e-2),
        "long": _long_rows_problem(),
        "mid": synth.sparse_text_logistic(500, 4099, mean_nnz=30.0, seed=3),
        # rcv1-like width (47,236 features): the gradient does not fit in LDS and is built in two column windows
        "wide": synth.sparse_text_logistic(1500, 47236, mean_nnz=75.0, seed=4),
        # the widest model whose gradient is one window in LDS (little room is left for staging entries: rows go in
        # small groups, and rows longer than the staging buffer straight from memory), and the first that takes two
        "lastone": synth.sparse_text_logistic(400, 35328, mean_nnz=120.0, seed=6),
        "firsttwo": synth.sparse_text_logistic(400, 35329, mean_nnz=120.0, seed=7),
        # the widest model the CSR kernels take (2^20 - 1 columns): about thirty column windows per worker step
        "widest": _widest_problem(),
    }


@pytest.fixture(scope="module")
def problems():
    return _problems()


def _model(rng, d, b_x, x_snap, spread=0.05):
    x = (x_snap + spread * rng.standard_normal(d)).astype(np.float32)
    if b_x == 32:
        return x.view(np.uint32).copy(), np.float32(1.0), x
    k, dx, _ = oracle.quantize(x, b_x, 3, 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    return oracle.pack(k, b_x), dx, oracle.dequantize(k, dx)


@pytest.mark.parametrize("name", ["text", "tiny", "long", "mid", "wide", "lastone", "firsttwo", "widest"])
def test_full_grad(dq, problems, name):
    p = problems[name]
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    x = (0.5 * np.random.default_rng(1).standard_normal(p.d)).astype(np.float32)
    g = torch.zeros(p.d, device="cuda")
    z = torch.zeros(p.n, device="cuda")
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = dq.new_workspace(dq.OP_FULL_GRAD, P)
    dq.dq_full_grad(P, dev(x), g, z, obj, ws)
    g_ref, z_ref = oracle.full_grad(rp, x, want_margins=True)
    _close(host(g), g_ref.astype(np.float64))
    _close(host(z), z_ref.astype(np.float64))
    assert abs(host(obj)[0] - oracle.objective(rp, x)) <= TOL * oracle.objective(rp, x)
    g2 = torch.zeros(p.d, device="cuda")
    dq.dq_full_grad(P, dev(x), g2, None, None, ws)
    assert torch.equal(g, g2)                      # deterministic


@pytest.mark.parametrize("have_z", [True, False])
@pytest.mark.parametrize("b_x", [8, 2, 32])
@pytest.mark.parametrize("name,M,B", [("text", 8, 32), ("tiny", 3, 5), ("long", 2, 40), ("mid", 4, 300), ("wide", 5, 48),
                                      ("lastone", 3, 40), ("firsttwo", 3, 40), ("widest", 2, 12)])
def test_vr_grad(dq, problems, name, M, B, b_x, have_z):
    p = problems[name]
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    d, n = p.d, p.n
    rng = np.random.default_rng(5)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, q = _model(rng, d, b_x, x_snap)
    idx = np.stack([oracle.sample_indices(n, B, 11, 2, w) for w in range(M)])
    if name == "long":
        idx[:, :6] = [3, 7, 8, 9, 3, 20]            # make sure the long rows are in the batch
    z_snap = None
    if have_z:
        _, z_ref = oracle.full_grad(rp, x_snap, want_margins=True)
        z_snap = dev(z_ref)
    ld = (d + 3) // 4 * 4
    alpha = torch.full((M, ld), 5.0, device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    l1n = torch.zeros(M, device="cuda")
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)          # a row per worker (wide gradients; split sparsifier)
    dq.dq_vr_grad(P, dev(idx), M, B, dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), b_x, False,
                  dev(x_snap), z_snap, alpha, amax, l1n, ws)
    for w in range(M):
        want = oracle.vr_grad(rp, idx[w], q, x_snap).astype(np.float64)
        got = host(alpha)[w]
        _close(got, want)
        assert host(amax)[w] == np.abs(got).max()
        assert abs(host(l1n)[w] - np.abs(got.astype(np.float64)).sum()) <= 1e-6 * np.abs(got).sum()
    # deterministic
    alpha2 = torch.zeros((M, ld), device="cuda")[:, :d]
    dq.dq_vr_grad(P, dev(idx), M, B, dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), b_x, False,
                  dev(x_snap), z_snap, alpha2, amax, None, ws)
    assert torch.equal(alpha, alpha2)


def _csr(rows, d, y=None, l2=1e-3, l1=1e-4):
    """Problem from a list of (columns, values) rows."""
    n = len(rows)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum([len(c) for c, _ in rows], out=indptr[1:])
    indices = np.concatenate([np.asarray(c, dtype=np.int32) for c, _ in rows])
    values = np.concatenate([np.asarray(v, dtype=np.float32) for _, v in rows])
    if y is None:
        y = np.where(np.arange(n) % 3 == 0, -1.0, 1.0).astype(np.float32)
    return synth.Problem(n=n, d=d, y=y, l2=l2, l1=l1, indptr=indptr, indices=indices, values=values)


def _vr_grad_case(dq, p, M, B, idx, spread, b_x=8):
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    d = p.d
    rng = np.random.default_rng(12)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, q = _model(rng, d, b_x, x_snap, spread=spread)
    _, z_ref = oracle.full_grad(rp, x_snap, want_margins=True)
    ld = (d + 3) // 4 * 4
    alpha = torch.zeros((M, ld), device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    dq.dq_vr_grad(P, dev(idx.astype(np.int32)), M, B, dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), b_x,
                  False, dev(x_snap), dev(z_ref), alpha, amax, None, ws)
    return host(alpha), [oracle.vr_grad(rp, idx[w].astype(np.int32), q, x_snap).astype(np.float64) for w in range(M)]


@pytest.mark.parametrize("spread", [0.05, 1e-4])
def test_vr_grad_many_rows_meet_in_one_column(dq, spread):
    """Every row of a 700-row mini-batch (three passes of the kernel over its rows) has columns 7 and 4098 next to a few
    others, with signs that cancel: the sums of those columns are built from 700 terms each, far below the bound the
    fixed-point unit of the accumulator is derived from -- with the model close to the snapshot (small coefficients) as
    well as far from it.  The tolerance stays 1e-5 of the largest entry."""
    rng = np.random.default_rng(3)
    d, n = 4101, 900
    rows = []
    for i in range(n):
        extra = np.sort(rng.choice(np.arange(8, 4098), size=rng.integers(0, 6), replace=False))
        cols = np.concatenate([[7], extra, [4098]])
        vals = rng.standard_normal(cols.size) * 0.3
        vals[0] = 0.5 * (1 if i % 2 else -1)
        rows.append((cols, vals))
    p = _csr(rows, d)
    idx = np.stack([rng.permutation(n)[:700] for _ in range(2)])
    got, want = _vr_grad_case(dq, p, 2, 700, idx, spread)
    for w in range(2):
        _close(got[w], want[w])


def test_vr_grad_values_of_very_different_size(dq):
    """Rows whose values differ by twelve orders of magnitude, the largest ones arriving in the last of three passes:
    the accumulator is rescaled to a coarser unit on the way and the result keeps the tolerance (relative to the
    largest entry of the gradient)."""
    rng = np.random.default_rng(4)
    d, n = 5000, 600
    rows = []
    for i in range(n):
        cols = np.sort(rng.choice(d, size=rng.integers(1, 40), replace=False))
        scale = 10.0 ** (-9 + 12 * i / n)
        rows.append((cols, rng.standard_normal(cols.size) * scale))
    p = _csr(rows, d)
    idx = np.stack([np.arange(n)])                   # in order: the large values come last
    got, want = _vr_grad_case(dq, p, 1, n, idx, 0.05)
    _close(got[0], want[0])


def test_a_value_that_is_not_a_number_poisons_its_worker_only(dq):
    """One NaN among the matrix values: the gradient of the worker whose mini-batch holds that row is NaN throughout,
    its largest magnitude is reported as NaN, and the fused step raises the status flag; the other worker is exact."""
    p0 = synth.sparse_text_logistic(300, 4099, mean_nnz=30.0, seed=3)
    values = p0.values.copy()
    bad_row = 17
    values[p0.indptr[bad_row] + 1] = np.nan
    p = synth.Problem(n=p0.n, d=p0.d, y=p0.y, l2=p0.l2, l1=p0.l1, indptr=p0.indptr, indices=p0.indices, values=values)
    M, B = 2, 20
    idx = np.stack([np.arange(0, B), np.arange(100, 100 + B)])           # worker 0 holds the row, worker 1 does not
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p0)
    d = p.d
    rng = np.random.default_rng(12)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, q = _model(rng, d, 8, x_snap)
    ld = (d + 3) // 4 * 4
    alpha = torch.zeros((M, ld), device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    xq_d, dx_d, xs_d = dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), dev(x_snap)
    dq.dq_vr_grad(P, dev(idx.astype(np.int32)), M, B, xq_d, dx_d, 8, False, xs_d, None, alpha, amax, None, ws)
    assert np.isnan(host(alpha)[0]).all() and np.isnan(host(amax)[0])
    _close(host(alpha)[1], oracle.vr_grad(rp, idx[1].astype(np.int32), q, x_snap).astype(np.float64))
    nw = dq.packed_words(d, 8)
    packed = torch.zeros((M, (nw + 3) // 4 * 4), dtype=torch.int32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    dq.dq_worker_step(P, dev(idx.astype(np.int32)), M, B, xq_d, dx_d, 8, False, xs_d, None, False, 8, 5, 1, 0, packed, delta,
                      None, None, status, ws)
    assert host(status)[0] & 1 and np.isnan(host(delta)[0]) and np.isfinite(host(delta)[1])


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_vr_grad_and_full_grad_on_random_shapes(dq, seed):
    """Forty seeded problems per seed whose shape is drawn at random: 1 to 36,001 columns (one, two, three columns; a
    ragged last quad; one and two column windows), rows of 0.3 to 80 entries on average with up to nine in ten
    rows empty, mini-batches of 1 to 600 rows (up to three passes), model widths 3, 4, 8, 11 and 32 bits, with and
    without cached margins, the model 0.05 to 1e-5 from the snapshot.  Variance-reduced and full gradient against
    the oracle."""
    rng = np.random.default_rng(seed)
    for case in range(40):
        d = int(rng.choice([1, 2, 3, 5, 17, 64, 100, 1000, 4099, 20958, 33000, 36001]))
        n = int(rng.integers(1, 400))
        mean = min(float(rng.choice([0.3, 1.0, 3.0, 20.0, 80.0])), d)
        lens = np.minimum(rng.poisson(mean, size=n), d)
        lens[rng.random(n) < float(rng.choice([0.0, 0.3, 0.9]))] = 0
        if lens.sum() == 0:
            lens[0] = 1
        rows = []
        for l in lens:
            cols = np.sort(rng.choice(d, size=l, replace=False))
            rows.append((cols, rng.standard_normal(l) * 10.0 ** rng.uniform(-3, 0) / np.sqrt(max(l, 1))))
        y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
        p = _csr(rows, d, y=y, l2=float(10.0 ** rng.uniform(-5, -2)))
        M, B = int(rng.integers(1, 6)), int(rng.choice([1, 3, 17, 64, 200, 300, 600]))
        b_x = int(rng.choice([8, 8, 4, 3, 11, 32]))
        P = dq.DeviceProblem.from_host(p)
        rp = oracle.RefProblem(p)
        x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
        x = (x_snap + float(rng.choice([0.05, 1e-3, 1e-5])) * rng.standard_normal(d)).astype(np.float32)
        if b_x == 32:
            xq, dx, q = x.view(np.uint32).copy(), np.float32(1.0), x
        else:
            k, dx, _ = oracle.quantize_wide(x, b_x, 3, 1, oracle.MASTER_ID, oracle.TAG_MODEL)
            xq, q = oracle.pack_wide(k, b_x), oracle.dequantize_wide(k, dx)
        idx = rng.integers(0, n, size=(M, B)).astype(np.int32)
        z_snap = None
        if rng.random() < 0.6:
            z_snap = dev(oracle.full_grad(rp, x_snap, want_margins=True)[1])
        ld = (d + 3) // 4 * 4
        alpha = torch.full((M, ld), 5.0, device="cuda")[:, :d]
        amax = torch.zeros(M, device="cuda")
        ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
        dq.dq_vr_grad(P, dev(idx), M, B, dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32)), b_x, False,
                      dev(x_snap), z_snap, alpha, amax, None, ws)
        for w in range(M):
            _close(host(alpha)[w], oracle.vr_grad(rp, idx[w], q, x_snap).astype(np.float64))
        g = torch.zeros(d, device="cuda")
        dq.dq_full_grad(P, dev(x), g, None, None, dq.new_workspace(dq.OP_FULL_GRAD, P))
        _close(host(g), oracle.full_grad(rp, x).astype(np.float64))


@pytest.mark.parametrize("sparsify", [False, True])
@pytest.mark.parametrize("b", [8, 4])
@pytest.mark.parametrize("name,M,B", [("text", 16, 64), ("tiny", 2, 7), ("long", 2, 12), ("wide", 4, 40), ("lastone", 3, 33),
                                      ("firsttwo", 3, 33), ("widest", 2, 9)])
def test_worker_step(dq, problems, name, M, B, b, sparsify):
    p = problems[name]
    P = dq.DeviceProblem.from_host(p)
    rp = oracle.RefProblem(p)
    d, n = p.d, p.n
    rng = np.random.default_rng(6)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, q = _model(rng, d, 8, x_snap)
    seed, it, w0 = 77, 9, 100
    idx = np.stack([oracle.sample_indices(n, B, seed, it, w0 + w) for w in range(M)])
    xs_d, xq_d, dx_d = dev(x_snap), dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32))
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    ld = (d + 3) // 4 * 4
    # fused, sampling inside the kernel
    packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    nnz = torch.zeros(M, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    alpha_f = torch.zeros((M, ld), device="cuda")[:, :d]
    ws = dq.new_workspace(dq.OP_VR_GRAD, P, M, B)
    dq.dq_worker_step(P, None, M, B, xq_d, dx_d, 8, False, xs_d, None, sparsify, b, seed, it, w0, packed, delta, nnz,
                      alpha_f, status, ws)
    # unfused chain of the same library with explicit indices: bit for bit
    alpha = torch.zeros((M, ld), device="cuda")[:, :d]
    amax = torch.zeros(M, device="cuda")
    dq.dq_vr_grad(P, dev(idx), M, B, xq_d, dx_d, 8, False, xs_d, None, alpha, amax, None, ws)
    assert torch.equal(alpha, alpha_f)
    v = alpha
    if sparsify:
        beta = torch.zeros((M, ld), device="cuda")[:, :d]
        kept = torch.zeros(M, dtype=torch.int32, device="cuda")
        dq.dq_sparsify(alpha, None, seed, it, w0, beta, amax, kept)
        v = beta
    packed2 = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    delta2 = torch.zeros(M, device="cuda")
    dq.dq_quantize_pack(v, b, amax, True, seed, it, dq.TAG_GRAD, w0, packed2, delta2)
    assert torch.equal(packed[:, :nw], packed2[:, :nw]) and torch.equal(delta, delta2)
    assert np.all(words(packed)[:, nw:] == 0xFFFFFFFF) and host(status)[0] == 0
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
        flips += int(np.count_nonzero(diff))
        if not sparsify:
            assert diff.max() <= 1
    assert flips <= max(3, 2e-3 * M * d), flips
    # the direct check: the oracle's sparsifier and quantizer applied to the gradient the GPU itself computed give
    # the GPU's message word for word (identical quantizer inputs => identical codes, no flips)
    for w in range(M):
        a_gpu = host(alpha_f)[w]
        v_o = oracle.sparsify(a_gpu, seed, it, w0 + w)[0] if sparsify else a_gpu
        k_o, d_o, _ = oracle.quantize(v_o, b, seed, it, w0 + w)
        assert host(delta)[w] == d_o
        assert np.array_equal(words(packed)[w, :nw], oracle.pack(k_o, b))
        assert host(nnz)[w] == np.count_nonzero(k_o)


def test_flag_bit_round_and_limits(dq, problems):
    p = problems["tiny"]
    P = dq.DeviceProblem.from_host(p)
    M, B, d = 2, 4, p.d
    packed = torch.full((M, 16), -1, dtype=torch.int32, device="cuda")
    delta = torch.full((M,), 3.0, device="cuda")
    dq.dq_worker_step(P, None, M, B, None, None, 8, True, torch.zeros(d, device="cuda"), None, True, 4, 1, 1, 0,
                      packed, delta, None, None, None, None)
    assert not words(packed)[:, : dq.packed_words(d, 4)].any() and not host(delta).any()
    # more columns than the staged entries can address: refused, not mangled
    wide = 1 << 20
    big = synth.Problem(n=2, d=wide, y=np.ones(2, dtype=np.float32), l2=0.0, l1=0.0,
                        indptr=np.array([0, 1, 2], dtype=np.int64), indices=np.array([0, 5], dtype=np.int32),
                        values=np.ones(2, dtype=np.float32))
    Pb = dq.DeviceProblem.from_host(big)
    x = torch.zeros(wide, device="cuda")
    with pytest.raises(dq.DqError) as e:
        dq.dq_full_grad(Pb, x, x.clone(), None, None, torch.zeros(1 << 22, device="cuda"))
    assert e.value.code == dq.ERR_UNSUPPORTED
    # a gradient that does not fit on chip needs the worker workspace
    pw = problems["wide"]
    Pw = dq.DeviceProblem.from_host(pw)
    # (a row per worker, slice results, one row for dq_run_rounds, and its two sets of prepared mini-batches: per
    # worker 1288 words and a pair of words for each of at most 8192 staged entries)
    row = (pw.d + 3) // 4 * 4 * 4
    need = dq.dq_workspace_bytes(dq.OP_VR_GRAD, Pw, 3, 4)
    assert 3 * row + 3 * 8 * 8 + row + 2 * 3 * 1288 * 4 < need <= 3 * row + 3 * 8 * 8 + row + 2 * 3 * (1288 + 2 * 8192) * 4
    with pytest.raises(dq.DqError) as e:
        dq.dq_worker_step(Pw, None, 3, 4, torch.zeros(pw.d, dtype=torch.int32, device="cuda"), torch.ones(1, device="cuda"),
                          8, False, torch.zeros(pw.d, device="cuda"), None, False, 8, 1, 1, 0,
                          torch.zeros((3, 11812), dtype=torch.int32, device="cuda"), torch.zeros(3, device="cuda"),
                          None, None, None, None)
    assert e.value.code == dq.ERR_WORKSPACE


@pytest.mark.parametrize("sparsify", [False, True])
@pytest.mark.parametrize("b", [8, 4, 2])
def test_worker_step_without_nonzero_counts_uses_several_blocks_per_worker(dq, problems, b, sparsify):
    """Without nnz_out the final quantization of a worker is shared by several identical blocks: same bits."""
    p = problems["text"]
    P = dq.DeviceProblem.from_host(p)
    d, n = p.d, p.n
    M, B = 5, 40
    rng = np.random.default_rng(8)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, _ = _model(rng, d, 8, x_snap)
    xs_d, xq_d, dx_d = dev(x_snap), dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32))
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    outs = []
    for want_nnz in (True, False):
        packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
        delta = torch.zeros(M, device="cuda")
        nnz = torch.zeros(M, dtype=torch.int32, device="cuda") if want_nnz else None
        dq.dq_worker_step(P, None, M, B, xq_d, dx_d, 8, False, xs_d, None, sparsify, b, 5, 6, 7, packed, delta, nnz,
                          None, None, None)
        outs.append((packed, delta))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert np.all(words(outs[1][0])[:, nw:] == 0xFFFFFFFF)


@pytest.mark.parametrize("sparsify,b,want_nnz", [(True, 8, True), (True, 4, True), (True, 4, False), (True, 2, False),
                                                  (False, 8, False), (False, 4, False), (False, 2, False)])
@pytest.mark.parametrize("M,B", [(5, 40), (16, 64), (3, 300)])
def test_worker_step_with_and_without_workspace(dq, problems, sparsify, b, want_nnz, M, B):
    """With a workspace and few workers, the identical blocks of a worker sparsify one slice each into memory and a
    second launch quantizes with the scale taken from the slices' maxima; without one (and without the sparsifier)
    the step is a single launch.  Same packed words, scales and kept counts either way, the oracle's counts, and
    the same gradient when it is asked for."""
    p = problems["text"]
    P = dq.DeviceProblem.from_host(p)
    d = p.d
    rng = np.random.default_rng(80 + b)
    x_snap = (0.3 * rng.standard_normal(d)).astype(np.float32)
    xq, dx, _ = _model(rng, d, 8, x_snap)
    xs_d, xq_d, dx_d = dev(x_snap), dev(xq.view(np.int32)), dev(np.array([dx], dtype=np.float32))
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    outs = []
    # (a workspace for a run of rounds, one of the size a single step needs, none)
    assert 0 < dq.dq_workspace_bytes(dq.OP_WORKER_STEP, P, M, B) < dq.dq_workspace_bytes(dq.OP_VR_GRAD, P, M, B)
    for ws in (dq.new_workspace(dq.OP_VR_GRAD, P, M, B), dq.new_workspace(dq.OP_WORKER_STEP, P, M, B), None):
        packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
        delta = torch.zeros(M, device="cuda")
        nnz = torch.full((M,), -7, dtype=torch.int32, device="cuda") if want_nnz else None
        alpha = torch.full((M, (d + 3) // 4 * 4), 9.0, device="cuda")[:, :d]
        dq.dq_worker_step(P, None, M, B, xq_d, dx_d, 8, False, xs_d, None, sparsify, b, 5, 6, 7, packed, delta, nnz,
                          alpha, None, ws)
        outs.append((packed, delta, nnz, alpha))
    for other in outs[1:]:
        assert torch.equal(outs[0][0], other[0]) and torch.equal(outs[0][1], other[1])
        assert torch.equal(outs[0][3], other[3])
        if want_nnz:
            assert torch.equal(outs[0][2], other[2])
    assert np.all(words(outs[0][0])[:, nw:] == 0xFFFFFFFF)
    assert host(outs[0][1]).all()                                       # every worker has a nonzero scale
    if want_nnz:
        codes = np.stack([oracle.unpack(words(outs[0][0])[w, :nw], d, b) for w in range(M)])
        assert np.array_equal(host(outs[0][2]), np.count_nonzero(codes, axis=1))
