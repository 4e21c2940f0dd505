"""GPU parity of whole rounds and epochs (Alg. 1-3) against the oracle's loops.

Two protocols.  Lock-step: before every round the GPU state is overwritten with the
oracle's, the GPU runs the round, and its outputs are compared with the oracle's round
(codes up to decisions flipped by sub-tolerance differences of alpha; the new model to
1e-5).  Free run: both sides run whole epochs independently from the same seed and the
objectives at the snapshots are compared.
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


def _trainer(dq, p, cfg, m, seed):
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    P = dq.DeviceProblem.from_host(p)
    return DoubleQuantTrainer(P, cfg.algo, cfg.M, cfg.B, cfg.b_x, cfg.b, m, cfg.lr, seed=seed)


def _small(cfg_name):
    cfg = synth.CONFIGS[cfg_name]
    if cfg_name == "C1":
        return cfg, synth.make_problem(cfg), 40
    if cfg_name == "C4":
        return cfg, synth.make_problem(cfg, n=3000), 6
    return cfg, synth.make_problem(cfg, n=4000), 12


@pytest.mark.parametrize("name", ["C1", "C4", "C2", "C3"])
def test_lock_step_rounds(dq, name):
    cfg, p, m = _small(name)
    seed = 3
    tr = _trainer(dq, p, cfg, m, seed)
    rp = oracle.RefProblem(p)
    d, M, B, b, bx = p.d, cfg.M, cfg.B, cfg.b, cfg.b_x
    acc = cfg.algo == "acc"
    x_snap = np.zeros(d, dtype=np.float32)
    y = x_snap.copy()
    flips = total = 0
    for e in range(2):
        # ---- oracle epoch start
        if acc:
            theta = np.float32(2.0 / (e + 3))
            eta = np.float32(np.float32(cfg.lr) / theta)
            x = oracle.acc_mix(y, x_snap, theta)
            xsum = np.zeros(d, dtype=np.float32)
        else:
            theta, eta = np.float32(0), np.float32(cfg.lr)
            x = x_snap.copy()
        g_snap = oracle.full_grad(rp, x_snap)
        # ---- GPU epoch start from the oracle's state
        tr.epoch_index = e
        tr.x_snap.copy_(dev(x_snap)); tr.y.copy_(dev(y))
        tr.epoch_prologue()
        assert np.abs(host(tr.g_snap) - g_snap).max() <= TOL * np.abs(g_snap).max()
        assert np.array_equal(host(tr.x), x)
        for t in range(m):
            it = e * m + t
            q, xq_words, dx, bits = alg.model_message(x, x_snap, bx, seed, it)
            flag = bits == 1
            # overwrite the GPU state with the oracle's
            tr.x.copy_(dev(x)); tr.g_snap.copy_(dev(g_snap))
            if acc:
                tr.y.copy_(dev(y)); tr.xsum.copy_(dev(xsum))
            if not flag:
                tr.xq[: xq_words.size].copy_(dev(xq_words.view(np.int32)))
                tr.delta_x.copy_(dev(np.array([dx], dtype=np.float32)))
            assert tr.round(t) == flag
            # ---- oracle round
            codes = np.zeros((M, d), dtype=np.int8)
            deltas = np.zeros(M, dtype=np.float32)
            for w in range(M):
                wd, dl, _, _, _, _ = alg.worker_message(rp, q, x_snap, flag, B, b, seed, it, w, cfg.algo == "sparse")
                codes[w] = oracle.unpack(wd, d, b)
                deltas[w] = dl
            if acc:
                oracle.master_update(codes, deltas, np.float32(1.0 / M), g_snap, x, y, x_snap, xsum, eta=eta,
                                     theta=theta, l1=rp.l1)
            else:
                oracle.master_update(codes, deltas, np.float32(1.0 / M), g_snap, x, eta=eta, l1=rp.l1)
            # ---- compare the round
            got_codes = np.stack([oracle.unpack(words(tr.packed)[w], d, b) for w in range(M)])
            diff = np.abs(got_codes.astype(np.int32) - codes)
            assert diff.max() <= 1
            flips += int(diff.sum()); total += diff.size
            assert np.all(np.abs(host(tr.delta) - deltas) <= 2e-5 * deltas + 1e-30)
            scale = max(np.abs(x).max(), 1e-30)
            # a flipped code moves a coordinate by eta*delta/M; everything else agrees to rounding
            bound = TOL * scale + float(eta) * float(deltas.max()) / M * (diff.max(axis=0) > 0)
            assert np.all(np.abs(host(tr.x) - x) <= bound + 1e-7 * scale)
        if acc:
            x_snap = oracle.acc_snapshot(xsum, m)
        else:
            x_snap = x.copy()
        tr.x.copy_(dev(x))
        if acc:
            tr.xsum.copy_(dev(xsum)); tr.y.copy_(dev(y))
        tr.epoch_epilogue()
        assert np.array_equal(host(tr.x_snap), x_snap)
    assert flips <= max(2, 1e-3 * total), (flips, total)


@pytest.mark.parametrize("name", ["C1", "C4", "C2", "C3"])
def test_free_run_objectives(dq, name):
    cfg, p, m = _small(name)
    S = 2
    tr = _trainer(dq, p, cfg, m, seed=0)
    log = tr.run(S)
    ref = alg.run(p, cfg.algo, cfg.M, cfg.B, cfg.b_x, cfg.b, m, S, cfg.lr, seed=0)
    assert len(log.objectives) == len(ref.objectives) == S + 1
    for a, b in zip(log.objectives, ref.objectives):
        assert abs(a - b) <= TOL * abs(b), (log.objectives, ref.objectives)
    assert log.objectives[-1] < log.objectives[0]
    assert log.bits_up == ref.bits_up and log.bits_down == ref.bits_down
    rel = np.abs(host(tr.x_snap) - ref.x_snap).max() / np.abs(ref.x_snap).max()
    assert rel < 1e-3, rel       # free-running trajectories differ by a few flipped roundings


def test_flag_bit_rule_when_an_update_leaves_the_model_at_the_snapshot(dq):
    """Section 4.1 sends one flag bit when the model equals the snapshot.  The library decides that from where a round
    stands in the epoch (first round of an epoch that starts at the snapshot); the oracle compares the two vectors bit
    for bit at every round.  The two rules part only when an update returns the model to the snapshot exactly -- here a
    prox that zeroes every step from a zero start.  What must hold then: the same iterates and gradient messages
    (the quantized model of an all-zero vector is the snapshot itself, so the workers' gradients vanish either way),
    and a download count that differs by exactly the model messages the library sends where the oracle sends flags."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    n, d, M, B, m, S = 400, 256, 4, 8, 6, 2
    p = synth.dense_logistic(n, d, seed=4, l2=1e-4, l1=10.0)          # l1 far above any gradient entry: prox gives 0
    tr = DoubleQuantTrainer(dq.DeviceProblem.from_host(p), "asylpg", M, B, 8, 8, m, 0.1, seed=2)
    log = tr.run(S)
    ref = alg.run(p, "asylpg", M, B, 8, 8, m, S, 0.1, seed=2)
    assert not host(tr.x).any() and not ref.x.any()                    # the model never leaves the snapshot
    assert not host(tr.delta).any() and not words(tr.packed).any()     # all-zero gradient messages, scale 0
    for a, b in zip(log.objectives, ref.objectives):
        assert abs(a - b) <= TOL * abs(b)
    assert log.bits_up == ref.bits_up
    assert ref.bits_down == S * m                                      # the oracle: a flag bit every round
    assert log.bits_down == S * (1 + (m - 1) * (32 + 8 * d))           # the library: a flag at the epoch start only


def test_runs_are_reproducible(dq):
    cfg, p, m = _small("C1")
    a = _trainer(dq, p, cfg, 10, seed=5); a.run(2)
    b = _trainer(dq, p, cfg, 10, seed=5); b.run(2)
    c = _trainer(dq, p, cfg, 10, seed=6); c.run(2)
    assert torch.equal(a.x_snap, b.x_snap) and torch.equal(a.packed, b.packed)
    assert not torch.equal(a.x_snap, c.x_snap)


@pytest.mark.parametrize("algo,b,d,M,B,b_x", [("acc", 8, 4096, 32, 256, 8), ("asylpg", 4, 4096, 16, 64, 8),
                                              ("sparse", 4, 3000, 8, 128, 8), ("acc", 2, 2048, 32, 128, 8),
                                              ("asylpg", 8, 1500, 4, 64, 8), ("asylpg", 8, 4096, 8, 64, 4),
                                              ("acc", 4, 2048, 16, 64, 2), ("acc", 8, 8192, 8, 32, 8),
                                              ("asylpg", 8, 6004, 8, 16, 4), ("acc", 8, 4096, 32, 256, 11)])
def test_rounds_enqueued_together_equal_rounds_enqueued_one_by_one(dq, algo, b, d, M, B, b_x):
    """How the rounds of an epoch are spread over dq_run_rounds calls (3 + 4 rounds, or one round per call) must not
    matter: every vector and every message comes out identical, bit for bit.  (Between the rounds of one call the
    model is quantized by the next round's row-streaming kernel instead of the master's: one round per call never
    takes that path, several rounds per call do wherever the shape allows it.)"""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    p = synth.dense_logistic(600, d, seed=d + M, l2=1e-3)
    P = dq.DeviceProblem.from_host(p)
    m = 7
    runs = []
    for together in (True, False):
        tr = DoubleQuantTrainer(P, algo, M, B, b_x, b, m, 0.1, seed=9)
        for _ in range(2):
            tr.epoch_prologue()
            if together:
                tr.rounds(0, 3)
                tr.rounds(3, m - 3)
            else:
                for t in range(m):
                    tr.rounds(t, 1)
            tr.epoch_epilogue()
        torch.cuda.synchronize()
        runs.append(tr)
    a, c = runs
    for name in ("x", "x_snap", "packed", "delta", "xq", "delta_x", "absmax_x"):
        assert torch.equal(getattr(a, name), getattr(c, name)), name
    if algo == "acc":
        assert torch.equal(a.y, c.y) and torch.equal(a.xsum, c.xsum)
    assert np.isfinite(host(a.x)).all() and host(a.x).any()


@pytest.mark.parametrize("algo,b,M,B,b_x,cache", [
    ("asylpg", 8, 8, 32, 8, True), ("sparse", 4, 16, 64, 8, True), ("asylpg", 4, 3, 20, 4, True),
    ("sparse", 8, 40, 16, 2, True), ("asylpg", 8, 8, 32, 11, True),
    ("asylpg", 8, 4, 88, 8, True),        # about 4500 entries per mini-batch: more than a thread stages in one go
    ("asylpg", 8, 2, 128, 8, True),       # about 6500: more than the staging buffer holds, nothing is prepared ahead
    ("asylpg", 8, 2, 300, 8, True),       # more rows than one pass takes
    ("sparse", 4, 64, 8, 8, True),        # many workers: one block each
    ("asylpg", 8, 8, 32, 8, False), ("sparse", 4, 16, 64, 8, False),     # margins at the snapshot recomputed
    ("asylpg", 8, 4, 88, 8, False),       # ... with their smaller staging buffer: not prepared ahead
    ("acc", 8, 8, 32, 8, True), ("acc", 4, 16, 64, 4, True)])            # Alg. 3 on the same features
def test_rounds_enqueued_together_equal_rounds_enqueued_one_by_one_sparse_features(dq, algo, b, M, B, b_x, cache):
    """The same for CSR features (the shape of configs C2 and C3).  With several rounds per call the master leaves
    (decoded model) - snapshot for the next round's workers, may quantize the sparsified gradients itself, and every
    worker launch draws, reads and lays out the next round's mini-batches in blocks of its own; rounds enqueued one
    per call do none of that.  Messages, scales and iterates must agree bit for bit."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    p = synth.make_problem(synth.CONFIGS["C2"], n=3000)
    P = dq.DeviceProblem.from_host(p)
    m = 6
    runs = []
    for together in (True, False):
        tr = DoubleQuantTrainer(P, algo, M, B, b_x, b, m, 0.5, seed=4, cache_margins=cache)
        for _ in range(2):
            tr.epoch_prologue()
            if together:
                tr.rounds(0, 4)
                tr.rounds(4, m - 4)
            else:
                for t in range(m):
                    tr.rounds(t, 1)
            tr.epoch_epilogue()
        torch.cuda.synchronize()
        runs.append(tr)
    a, c = runs
    for name in ("x", "x_snap", "packed", "delta", "xq", "delta_x", "absmax_x", "nnz") + (("y", "xsum") if algo == "acc" else ()):
        assert torch.equal(getattr(a, name), getattr(c, name)), name
    assert np.isfinite(host(a.x)).all() and host(a.x).any() and host(a.status)[0] == 0


@pytest.mark.parametrize("b,M,each,b_x,counts", [(4, 16, False, 8, True), (8, 24, False, 8, True), (4, 5, True, 4, True),
                                                  (8, 32, True, 32, True), (2, 8, False, 8, True), (2, 8, False, 8, False),
                                                  (4, 20, False, 8, False)])
@pytest.mark.parametrize("shape", ["C3", "ragged"])
def test_master_that_quantizes_the_sparsified_gradients_equals_the_separate_steps(dq, b, M, each, b_x, counts, shape):
    """Alg. 2 on CSR features wide enough for the sparsifier to be split over several blocks per worker: inside
    dq_run_rounds the master kernel quantizes the workers' sparsified gradients while it aggregates them.  A round
    enqueued that way must leave messages, scales, nonzero counts, the model and the model's message bit for bit
    as dq_worker_step followed by dq_master_step do, which quantize in a launch of their own (M = 20, 24 and 32: more
    workers than one pass of the kernel takes; b = 2 with nonzero counts: the route is not taken, both sides are the
    separate steps; without counts (`nnz` null in the run state) 2-bit messages take it too)."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    # ("ragged": 4099 columns, the narrowest kind of model the route is taken for, its last quad one coordinate long)
    p = synth.make_problem(synth.CONFIGS["C3"], n=3000) if shape == "C3" else \
        synth.sparse_text_logistic(500, 4099, mean_nnz=30.0, seed=3)
    P = dq.DeviceProblem.from_host(p)
    B, m, seed = 32, 4, 9
    one = DoubleQuantTrainer(P, "sparse", M, B, b_x, b, m, 0.5, seed=seed, each=each)
    two = DoubleQuantTrainer(P, "sparse", M, B, b_x, b, m, 0.5, seed=seed, each=each)
    if not counts:
        one.state.nnz = None
        two.state.nnz = None
    one.epoch_prologue(); two.epoch_prologue()
    one.rounds(0, 3)
    idx = torch.empty(M * B, dtype=torch.int32, device="cuda")
    for t in range(3):
        if t == 0:
            two.rounds(0, 1)                               # (the model is the snapshot: all-zero messages)
            continue
        dq.dq_sample_indices(P.n, M, B, seed, t, 0, idx)
        dq.dq_worker_step(P, idx, M, B, two.xq, two.delta_x, b_x, False, two.x_snap, two.z_snap, True, b, seed, t, 0,
                          two.packed, two.delta, nnz_out=two.nnz[t] if counts else None, status=two.status, ws=two.ws)
        step = dq.dq_master_step_each if each else dq.dq_master_step
        args = (two.packed, two.delta, M, b) + (() if each else (float(np.float32(1) / np.float32(M)),))
        step(*args, two.g_snap, two.x, None, two.x_snap, None, two.eta, 0.0, P.l1, b_x, seed, t + 1,
             two.xq, two.delta_x, two.absmax_x[t & 1:], two.status)
    torch.cuda.synchronize()
    for name in ("packed", "delta", "nnz", "x", "xq", "delta_x", "status"):
        assert torch.equal(getattr(one, name), getattr(two, name)), name
    assert host(one.x).any() and host(one.packed).any() and host(one.status)[0] == 0
    assert host(one.nnz)[1:3].all() if counts else not host(one.nnz).any()


@pytest.mark.parametrize("name", ["C1", "C4", "C2"])
def test_kernel_events_time_the_worker_kernel_and_change_nothing(dq, name):
    """dq_run_rounds with worker_events: each pair receives the start and end of the row-streaming kernel's launch
    (a positive duration far below a millisecond on these sizes) and the round computes exactly what it computes
    without events."""
    cfg, p, m = _small(name)
    m = min(m, 6)
    a = _trainer(dq, p, cfg, m, seed=3)
    b = _trainer(dq, p, cfg, m, seed=3)
    a.epoch_prologue(); b.epoch_prologue()
    pairs = []
    for t in range(m):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); e1.record()                       # creates the HIP events
        a.rounds(t, 1, [e0.cuda_event, e1.cuda_event])
        pairs.append((e0, e1, a.is_flag_round(t)))
    b.rounds(0, m)
    torch.cuda.synchronize()
    assert torch.equal(a.x, b.x) and torch.equal(a.packed, b.packed) and torch.equal(a.delta, b.delta)
    timed = [e0.elapsed_time(e1) for e0, e1, flag in pairs if not flag]
    assert len(timed) >= m - 1
    assert all(1e-4 < ms < 1.0 for ms in timed), timed


@pytest.mark.parametrize("algo,b_x,b", [("asylpg", 32, 32), ("acc", 32, 32), ("asylpg", 32, 8), ("asylpg", 8, 32),
                                        ("sparse", 32, 4)])
def test_unquantized_modes_free_run(dq, algo, b_x, b):
    """b = 32 / b_x = 32: AsyFPG, Acc-AsyFPG and QSVRG-style runs through the same kernels."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    cfg = synth.CONFIGS["C1"]
    p = synth.make_problem(cfg, n=600, d=200)
    m, S = 12, 2
    tr = DoubleQuantTrainer(dq.DeviceProblem.from_host(p), algo, cfg.M, cfg.B, b_x, b, m, cfg.lr, seed=4)
    log = tr.run(S)
    ref = alg.run(p, algo, cfg.M, cfg.B, b_x, b, m, S, cfg.lr, seed=4)
    for a, r in zip(log.objectives, ref.objectives):
        assert abs(a - r) <= TOL * abs(r)
    assert log.bits_down == ref.bits_down
    if algo != "sparse":
        assert log.bits_up == ref.bits_up
    else:
        assert abs(log.bits_up - ref.bits_up) <= 0.01 * ref.bits_up      # a flipped keep decision moves a few codes
    rel = np.abs(host(tr.x_snap) - ref.x_snap).max() / np.abs(ref.x_snap).max()
    assert rel < (2e-5 if (b, b_x) == (32, 32) else 2e-3), rel


def test_comparison_of_the_six_algorithms(dq):
    from paper_1805_10111_amd.compare import run_comparison
    cfg = synth.CONFIGS["C1"]
    p = synth.make_problem(cfg, n=1000, d=400)
    res = run_comparison(cfg, p, epochs=3, threshold=0.69, b=8, m=40)
    assert set(res) == {"AsyFPG", "Acc-AsyFPG", "QSVRG", "AsyLPG", "Sparse-AsyLPG", "Acc-AsyLPG"}
    fp, lp, qs, sp = res["AsyFPG"], res["AsyLPG"], res["QSVRG"], res["Sparse-AsyLPG"]
    assert lp["bits_total"] < qs["bits_total"] < fp["bits_total"]
    assert sp["bits_total"] < lp["bits_total"]
    assert abs(lp["objectives"][-1] - fp["objectives"][-1]) < 0.01 * fp["objectives"][-1]
    assert 3.5 < fp["bits_total"] / lp["bits_total"] < 4.1        # (32 d) / (32 + 8 d) per message


def test_mu_trace_follows_the_papers_observation(dq):
    """Fig. 2 of the paper: the mu needed for condition (2) is largest right after the snapshot
    (x is still close to it) and falls as x moves away within the epoch."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    cfg = synth.CONFIGS["C1"]
    p = synth.make_problem(cfg, n=600, d=200)
    tr = DoubleQuantTrainer(dq.DeviceProblem.from_host(p), "asylpg", cfg.M, cfg.B, 8, 8, 30, cfg.lr, seed=1)
    tr.run_epoch(record_mu=True)
    tr.run_epoch(record_mu=True)
    assert len(tr.mu_trace) == 60
    # (in the very first epoch the snapshot is 0 and both sides scale with ||x||^2: the ratio is flat)
    mus = [r[2] / r[3] for r in tr.mu_trace if r[0] == 1 and r[3] > 0]
    assert all(np.isfinite(mus))
    assert mus[0] == max(mus) and mus[0] > 10 * mus[-1]


@pytest.mark.parametrize("name,algo,tau,b_x,b", [("C1", "asylpg", 1, 8, 8), ("C1", "asylpg", 3, 8, 8), ("C1", "acc", 2, 8, 8),
                                                 ("C1", "asylpg", 3, 32, 32), ("C2", "asylpg", 3, 8, 8), ("C3", "sparse", 5, 8, 4)])
def test_bounded_delay_free_run(dq, name, algo, tau, b_x, b):
    """Emulated staleness (Assumption 3): worker group g reads the model of g rounds ago."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    cfg = synth.CONFIGS[name]
    p = synth.make_problem(cfg, n=1500) if cfg.csr else synth.make_problem(cfg, n=600, d=200)
    m, S = 10, 2
    tr = DoubleQuantTrainer(dq.DeviceProblem.from_host(p), algo, cfg.M, cfg.B, b_x, b, m, cfg.lr, seed=2, tau=tau)
    log = tr.run(S)
    ref = alg.run(p, algo, cfg.M, cfg.B, b_x, b, m, S, cfg.lr, seed=2, tau=tau)
    sync = alg.run(p, algo, cfg.M, cfg.B, b_x, b, m, S, cfg.lr, seed=2)
    for a, r in zip(log.objectives, ref.objectives):
        assert abs(a - r) <= TOL * abs(r)
    rel = np.abs(host(tr.x_snap) - ref.x_snap).max() / np.abs(ref.x_snap).max()
    assert rel < 2e-3, rel
    # the delay is visible: the delayed trajectory differs from the synchronous one by more than that
    assert np.abs(ref.x_snap - sync.x_snap).max() / np.abs(ref.x_snap).max() > 5 * max(rel, 1e-6)
    assert log.bits_down == ref.bits_down


def test_delay_argument_checks(dq):
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    cfg = synth.CONFIGS["C1"]
    p = synth.make_problem(cfg, n=100, d=64)
    tr = DoubleQuantTrainer(dq.DeviceProblem.from_host(p), "asylpg", cfg.M, cfg.B, 8, 8, 4, cfg.lr, tau=cfg.M)
    with pytest.raises(dq.DqError) as e:          # at most one delay group per worker
        tr.run_epoch()
    assert e.value.code == dq.ERR_INVALID_ARG


@pytest.mark.parametrize("algo,b_x,b,tau", [("asylpg", 8, 8, 0), ("asylpg", 32, 32, 0), ("acc", 8, 8, 0), ("sparse", 8, 4, 0),
                                             ("asylpg", 8, 8, 3)])
def test_one_master_update_per_gradient_free_run(dq, algo, b_x, b, tau):
    """Alg. 1 taken literally at the master: every message is its own update; with tau = M - 1 on top, worker w
    computes on a model that is w rounds old -- the paper's asynchronous picture on one GPU."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    cfg = synth.CONFIGS["C1"]
    p = synth.make_problem(cfg, n=600, d=200)
    m, S, lr = 10, 2, 0.03
    tr = DoubleQuantTrainer(dq.DeviceProblem.from_host(p), algo, cfg.M, cfg.B, b_x, b, m, lr, seed=5, tau=tau, each=True)
    log = tr.run(S)
    ref = alg.run(p, algo, cfg.M, cfg.B, b_x, b, m, S, lr, seed=5, tau=tau, each=True)
    for a, r in zip(log.objectives, ref.objectives):
        assert abs(a - r) <= TOL * abs(r)
    assert log.bits_down == ref.bits_down
    mean_mode = alg.run(p, algo, cfg.M, cfg.B, b_x, b, m, S, lr, seed=5, tau=tau)
    assert abs(mean_mode.objectives[-1] - ref.objectives[-1]) > 1e-4          # the two aggregation rules differ


@pytest.mark.parametrize("algo,b", [("asylpg", 8), ("sparse", 4)])
def test_free_run_on_a_model_wider_than_the_on_chip_buffer(dq, algo, b):
    """rcv1-like width (47,236 features): the CSR worker builds its gradient in two column windows."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    p = synth.sparse_text_logistic(1500, 47236, mean_nnz=75.0, seed=4, l2=1e-4, l1=1e-5)
    M, B, m, S, lr = 4, 16, 6, 2, 0.1
    tr = DoubleQuantTrainer(dq.DeviceProblem.from_host(p), algo, M, B, 8, b, m, lr, seed=2)
    log = tr.run(S)
    ref = alg.run(p, algo, M, B, 8, b, m, S, lr, seed=2)
    for a, r in zip(log.objectives, ref.objectives):
        assert abs(a - r) <= TOL * abs(r)
    assert log.bits_down == ref.bits_down
    if algo == "asylpg":
        assert log.bits_up == ref.bits_up


def test_sparse_messages_through_the_wire_format(dq):
    """Alg. 2 with every message really encoded as (position, value) entries (Section 4.2) and decoded again
    before the master uses it: same trajectory bit for bit, and the entry counts are the ones the bit counter uses."""
    from paper_1805_10111_amd.driver import DoubleQuantTrainer
    cfg = synth.CONFIGS["C3"]
    p = synth.make_problem(cfg, n=3000)
    P = dq.DeviceProblem.from_host(p)
    m, S = 6, 2
    a = DoubleQuantTrainer(P, "sparse", cfg.M, cfg.B, cfg.b_x, cfg.b, m, cfg.lr, seed=3)
    b = DoubleQuantTrainer(P, "sparse", cfg.M, cfg.B, cfg.b_x, cfg.b, m, cfg.lr, seed=3, sparse_wire=True)
    la, lb = a.run(S), b.run(S)
    assert torch.equal(a.x_snap, b.x_snap) and la.bits_up == lb.bits_up and la.objectives == lb.objectives
    assert torch.equal(b.wire_nnz, b.nnz[m - 1])                       # entries of the last round's messages
    used = (host(b.wire_nnz).astype(np.int64) * (15 + cfg.b) + 31) // 32      # ceil(log2 20958) = 15 position bits
    w = words(b.wire)
    for r in range(cfg.M):
        assert not w[r, used[r]:].any() and (used[r] == 0 or w[r, :used[r]].any())


@pytest.mark.parametrize("name", ["C1", "C4", "C3"])
def test_rounds_replayed_from_a_captured_graph(dq, name):
    """dq_run_rounds only enqueues kernels (no allocation, no memset), so a caller may capture an epoch's rounds
    into a graph.  Every replay -- with eager work of the program between replays -- must give what the same
    rounds give when enqueued directly."""
    cfg, p, m = _small(name)
    m = min(m, 8)
    eager = _trainer(dq, p, cfg, m, seed=4)
    graph = _trainer(dq, p, cfg, m, seed=4)
    for tr in (eager, graph):
        tr.epoch_prologue()
        tr.rounds(0, m)                                  # warm-up: one-time function attributes are set outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            graph.rounds(0, m)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 16, device="cuda")
    for rep in range(3):
        eager.rounds(0, m)
        g.replay()
        scratch.add_(1.0)                                # the program's own eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(eager.x, graph.x) and torch.equal(eager.packed, graph.packed), rep
        assert torch.equal(eager.delta, graph.delta) and torch.equal(eager.xq, graph.xq), rep
    assert np.isfinite(host(graph.x)).all()
