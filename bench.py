#!/usr/bin/env python3
"""Benchmark of the double-quantization hot path on one MI355X.

A step is one synchronous round of the whole path for all M workers: model message ->
variance-reduced mini-batch gradients -> stochastic quantization -> packing -> master
decode/aggregate -> prox or momentum update -> model re-quantization.  The clock is a pair
of HIP events around every run of consecutive rounds; the epoch prologue (full gradient,
once per m rounds) runs at its real cadence but outside the clock and is reported apart.
Inputs are resident in HBM before the clock starts.

Prints ONE JSON line: worker-steps/s (= M * rounds / time of the round loop) on the
accelerated dense workload (config C4), the roofline figures of the dominant kernel from
the start/stop events of its own launches, the quantizer microbenchmark (config C5) as
extra fields, and the CPU oracle timed on bounded samples of the same workloads.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
EVENT_STRIDE = 4          # every EVENT_STRIDE-th round of the kernel-timing epochs carries launch events
KERNEL_EPOCHS = 8         # epochs run after the timed region for the dominant kernel's own duration
MIN_WARM_EPOCHS = 3       # whole epochs before the clock starts
MIN_TIMED_EPOCHS = 10     # epochs' worth of rounds that the reported median rests on
KERNEL_NAME = {False: "vr_dense_kernel (variance-reduced gradient, all M workers)",
               True: "csr_worker_kernel (whole worker step, all M workers)"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="C4", choices=["C1", "C2", "C3", "C4"])
    ap.add_argument("--n", type=int, default=None, help="override the number of samples (testing only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-quantizer", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) for calibrating profiler byte counters")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    return ap.parse_args()


def run_rounds(tr, rounds, loop_events=None, prologue_events=None):
    """Advance the trainer by `rounds` rounds, running epoch prologues/epilogues at their cadence.

    The round loop (Alg. 1-3, inner `for t`: model message, worker steps, master step) and the epoch prologue
    (full gradient at the snapshot) are timed apart: every contiguous run of rounds inside one epoch is bracketed
    by a pair of events appended to `loop_events` (the prologue and the epilogue lie outside every pair), and every
    prologue by a pair appended to `prologue_events`.
    """
    import torch

    def pair():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    done = 0
    while done < rounds:
        if tr._t == 0:
            if prologue_events is not None:
                p0, p1 = pair()
                p0.record()
            tr.epoch_prologue()
            if prologue_events is not None:
                p1.record()
                prologue_events.append((p0, p1))
        take = min(rounds - done, tr.m - tr._t)
        if loop_events is not None:
            e0, e1 = pair()
            e0.record()
        tr.rounds(tr._t, take)
        if loop_events is not None:
            e1.record()
            loop_events.append((e0, e1, take))
        tr._t += take
        done += take
        if tr._t == tr.m:
            tr.epoch_epilogue()
            tr._t = 0


def time_round_loop(tr, torch, steps, warmup):
    """Times the round loop (Alg. 1-3, inner `for t`) with events on the launch stream around whole runs of rounds;
    the epoch prologue (full gradient) and epilogue lie outside every bracket and are timed apart.  A measurement is
    `steps` consecutive rounds; it is repeated until at least MIN_TIMED_EPOCHS epochs' worth of rounds have been
    timed, and the caller reports the median measurement.  Warm-up: the `warmup` rounds asked for, and at least
    MIN_WARM_EPOCHS whole epochs.  Leaves the trainer at the start of an epoch."""
    m = tr.m
    run_rounds(tr, max(warmup, MIN_WARM_EPOCHS * m))
    torch.cuda.synchronize()
    repeats = max(1, -(-MIN_TIMED_EPOCHS * m // steps))
    per_repeat, prologue_events = [], []
    t0 = time.perf_counter()
    for _ in range(repeats):
        ev = []
        run_rounds(tr, steps, ev, prologue_events)
        per_repeat.append(ev)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if int(tr.status.item()) != 0:
        raise FloatingPointError("non-finite quantization scale during the benchmark")
    loop_s = sorted(sum(e0.elapsed_time(e1) for e0, e1, _ in ev) * 1e-3 for ev in per_repeat)
    prologues = sorted(p0.elapsed_time(p1) * 1e-3 for p0, p1 in prologue_events)
    while tr._t != 0:                   # finish the epoch that the last measurement ended in
        run_rounds(tr, 1)
    return {"loop_s": loop_s, "median_s": loop_s[len(loop_s) // 2], "repeats": repeats, "wall_s": wall,
            "prologues": prologues, "prologue_s": prologues[len(prologues) // 2] if prologues else None,
            "warm_rounds": max(warmup, MIN_WARM_EPOCHS * m)}


class _TimingEvents:
    """HIP events made for timing only (hipEventDisableSystemFence), straight from the HIP runtime the process already
    has loaded.  A launch whose stop event is an ordinary one ends with a system-scope release of the caches, which a
    plain launch does not, and reads about a microsecond longer; with this flag the launch that carries the events
    is the launch the timed region runs.  torch.cuda.Event cannot set the flag."""
    DISABLE_SYSTEM_FENCE = 0x20000000

    def __init__(self):
        import ctypes
        path = None
        for line in open("/proc/self/maps"):
            if "libamdhip64" in line:
                path = line.split()[-1]
                break
        if path is None:
            raise OSError("the HIP runtime is not loaded")
        self.C, self.hip, self.handles = ctypes, ctypes.CDLL(path), []

    def new(self):
        e = self.C.c_void_p()
        rc = self.hip.hipEventCreateWithFlags(self.C.byref(e), self.C.c_uint(self.DISABLE_SYSTEM_FENCE))
        if rc != 0:
            raise OSError(f"hipEventCreateWithFlags returned {rc}")
        self.handles.append(e)
        return e

    def elapsed_s(self, e0, e1):
        ms = self.C.c_float()
        rc = self.hip.hipEventElapsedTime(self.C.byref(ms), e0, e1)
        if rc != 0:
            raise OSError(f"hipEventElapsedTime returned {rc}")
        return ms.value * 1e-3

    def close(self):
        for e in self.handles:
            self.hip.hipEventDestroy(e)
        self.handles = []


def kernel_durations(tr, epochs, stride):
    """Own duration of the dominant kernel (the one that streams the feature rows of all M workers): in `epochs`
    further epochs, each enqueued by one call like the timed region, every `stride`-th round hands the library two
    events, which it uses as the start and stop events of that launch (hipExtLaunchKernel), i.e. the kernel's time
    stamps on the launch stream.  Flag-bit rounds read no rows and are skipped.  Returns seconds per launch (list)."""
    import torch
    ev = _TimingEvents()
    pairs = []
    for _ in range(epochs):
        assert tr._t == 0
        tr.epoch_prologue()
        handles = []
        for t in range(tr.m):
            if t % stride == stride - 1 and not tr.is_flag_round(t):
                e0, e1 = ev.new(), ev.new()
                pairs.append((e0, e1))
                handles += [e0.value, e1.value]
            else:
                handles += [None, None]
        tr.rounds(0, tr.m, handles)
        tr.epoch_epilogue()
    torch.cuda.synchronize()
    out = [ev.elapsed_s(e0, e1) for e0, e1 in pairs]
    ev.close()
    return out


def recorded_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter passes
    (profiles/traffic_<workload>.json), or None if the kernel's sources (the translation unit that holds it
    and the headers it includes, listed in the record) changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"traffic_{workload.lower()}.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    h = hashlib.sha256()
    try:
        for rel in rec["sources"]:
            h.update(open(os.path.join(ROOT, rel), "rb").read())
    except (KeyError, OSError):
        return None
    return rec["traffic_bytes_per_launch"] if rec.get("sources_sha256") == h.hexdigest() else None


def quantizer_leg(dq, torch):
    """Config C5: delta reduce, quantize+pack at b in {8,4,2}, decode-and-sum over M=16, on 2^28 coordinates."""
    import synth
    N, M = 1 << 28, 16
    v = torch.from_numpy(synth.mixture_vector(N, seed=0)).cuda()
    out = {}
    absmax = torch.zeros(1, device="cuda")
    delta = torch.zeros(M, device="cuda")

    def timed(fn, reps=5, groups=3):
        """Seconds per call: the median over `groups` measurements of `reps` back-to-back calls each."""
        fn(); torch.cuda.synchronize()
        per_call = []
        for _ in range(groups):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record(); torch.cuda.synchronize()
            per_call.append(e0.elapsed_time(e1) / reps * 1e-3)
        return sorted(per_call)[len(per_call) // 2]

    # what plain device kernels reach on the same box, for scale: a 1 GiB copy (read + write) and a 1 GiB read
    w = torch.empty_like(v)
    t = timed(lambda: w.copy_(v))
    out["plain_copy_1GiB"] = {"GB/s": round(2 * N * 4 / t * 1e-9, 1), "us": round(t * 1e6, 1)}
    del w
    t = timed(lambda: dq.dq_absmax(v, absmax))
    out["absmax"] = {"GB/s": round(N * 4 / t * 1e-9, 1), "us": round(t * 1e6, 1)}
    for b in (8, 4, 2):
        nw = dq.packed_words(N, b)
        packed = torch.zeros((M, nw), dtype=torch.int32, device="cuda")
        t = timed(lambda: dq.dq_quantize_pack(v, b, absmax, True, 0, 0, dq.TAG_GRAD, 3, packed[3], delta[3:4]))
        out[f"quantize_pack_b{b}"] = {"GB/s": round(N * (4 + b / 8) / t * 1e-9, 1), "us": round(t * 1e6, 1)}
        for w in range(M):
            dq.dq_quantize_pack(v, b, absmax, True, 0, 0, dq.TAG_GRAD, w, packed[w], delta[w:w + 1])
        res = torch.zeros(N, device="cuda")
        t = timed(lambda: dq.dq_unpack_dequant_sum(packed, delta, N, b, 1.0 / M, res))
        out[f"unpack_dequant_sum_b{b}_M16"] = {"GB/s": round(N * (M * b / 8 + 4) / t * 1e-9, 1), "us": round(t * 1e6, 1)}
        del packed, res
    for k in out:
        out[k]["frac_of_hbm_peak"] = round(out[k]["GB/s"] / HBM_PEAK_GBS, 3)
    return out


def graph_replay_us_per_round(tr, torch, rounds, repeats=10):
    """The rounds of one epoch captured once into a graph (dq_run_rounds only enqueues kernels) and replayed:
    microseconds per round, median over `repeats` replays timed with events on the replaying stream."""
    tr.epoch_prologue()
    tr.rounds(0, rounds)                                 # one-time kernel attributes are set outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            tr.rounds(0, rounds)
    torch.cuda.synchronize()
    times = []
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    times.sort()
    return times[len(times) // 2] / rounds * 1e3


def other_configs_leg(dq, torch, synth, Trainer, skip):
    """Rounds of the small, launch-bound configs (C1-C3): microseconds per round and worker-steps/s."""
    out = {}
    for name in ("C1", "C2", "C3"):
        if name == skip:
            continue
        cfg = synth.CONFIGS[name]
        prob = synth.make_problem(cfg)
        tr = Trainer(dq.DeviceProblem.from_host(prob), cfg.algo, cfg.M, cfg.B, cfg.b_x, cfg.b, cfg.m, cfg.lr, seed=cfg.seed)
        tr._t = 0
        rounds = cfg.m                              # a measurement = one epoch of rounds
        meas = time_round_loop(tr, torch, rounds, 0)
        dt = meas["median_s"]
        out[name] = {"us_per_round": round(dt / rounds * 1e6, 2), "worker_steps_per_s": round(cfg.M * rounds / dt, 1),
                     "rounds_per_measurement": rounds, "repeats": meas["repeats"], "M": cfg.M, "B": cfg.B, "d": prob.d,
                     "prologue_us": round(meas["prologue_s"] * 1e6, 1),
                     "us_per_round_graph_replay": round(graph_replay_us_per_round(tr, torch, rounds), 2),
                     "note": "launch/latency-bound: under 3 MB of traffic per round; round loop only, as `value`; "
                             "graph_replay: the same rounds captured once and replayed"}
        del tr
    return out


def cpu_baseline(cfg, prob, seconds):
    """The oracle, as it stands, on a bounded sample of the same workload: whole rounds for `seconds` on one
    thread, then for half as long with the M independent worker steps of a round spread over the host's cores
    (the oracle's C routines run outside the interpreter lock; nothing in the oracle changes for this)."""
    import numpy as np
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    from oracle import algorithms as alg
    rp = oracle.RefProblem(prob)
    d, M, B = prob.d, cfg.M, cfg.B
    sparse = cfg.algo == "sparse"

    def run(limit, pool):
        rng = np.random.default_rng(0)
        x_snap = (0.01 * rng.standard_normal(d)).astype(np.float32)
        x = (x_snap + 0.001 * rng.standard_normal(d)).astype(np.float32)
        g_snap = np.zeros(d, dtype=np.float32)
        y = x.copy()
        xsum = np.zeros(d, dtype=np.float32)
        t0 = time.perf_counter()
        rounds = 0
        while True:
            it = rounds + 1
            q, _, _, _ = alg.model_message(x, x_snap, cfg.b_x, 0, it)
            codes = np.zeros((M, d), dtype=np.int8)
            deltas = np.zeros(M, dtype=np.float32)

            def worker(w):
                wd, dl, *_ = alg.worker_message(rp, q, x_snap, False, B, cfg.b, 0, it, w, sparse)
                codes[w] = oracle.unpack(wd, d, cfg.b)
                deltas[w] = dl
            if pool is None:
                for w in range(M):
                    worker(w)
            else:
                list(pool.map(worker, range(M)))
            if cfg.algo == "acc":
                oracle.master_update(codes, deltas, np.float32(1 / M), g_snap, x, y, x_snap, xsum, eta=0.1, theta=0.5, l1=rp.l1)
            else:
                oracle.master_update(codes, deltas, np.float32(1 / M), g_snap, x, eta=0.1, l1=rp.l1)
            rounds += 1
            el = time.perf_counter() - t0
            if el >= limit:
                return rounds, el

    rounds, el = run(seconds, None)
    out = {"value": round(M * rounds / el, 2), "unit": "worker-steps/s", "cores": 1, "kind": "oracle",
           "sample": f"{rounds} rounds of {cfg.name} (M={M}, B={B}, d={d}; full gradient excluded), "
                     f"{el:.1f} s, single thread, gcc -O2"}
    threads = max(1, min(M, 16, len(os.sched_getaffinity(0))))
    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as pool:
            rounds, el = run(seconds / 2, pool)
        out["all_cores"] = {"value": round(M * rounds / el, 2), "unit": "worker-steps/s", "cores": threads,
                            "sample": f"{rounds} rounds, {el:.1f} s, the workers of a round on {threads} threads"}
    return out


def cpu_baseline_quantizer(log2n=24, M=16):
    """The oracle on config C5's three stages (scale reduction, quantize + pack, decode-and-sum over M messages) at
    b in {2, 4, 8}: GB/s of the same algorithmic bytes as the GPU figures, on a slice of 2^log2n coordinates of the
    same vector, on one thread and with contiguous chunks of the vector on all host threads (coordinates are
    independent and the random streams addressed, so chunking changes no result; a chunk draws its variates with the
    oracle's range generator and carries the global largest magnitude as one extra coordinate)."""
    import numpy as np
    import oracle
    import synth
    from concurrent.futures import ThreadPoolExecutor
    n = 1 << log2n
    v = synth.mixture_vector(n, seed=0)
    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    bounds = [n * i // threads // 32 * 32 for i in range(threads)] + [n]
    chunks = list(zip(bounds[:-1], bounds[1:]))
    out = {"unit": "GB/s", "kind": "oracle", "cores": [1, threads],
           "sample": f"the first 2^{log2n} of config C5's 2^28 coordinates, M={M} messages for the decode; each stage "
                     f"once on one thread and once with {threads} contiguous chunks on {threads} threads; gcc -O2"}

    def clock(fn):
        t0 = time.perf_counter()
        r = fn()
        return time.perf_counter() - t0, r

    def both(name, nbytes, one, chunked, pool):
        t1, r1 = clock(one)
        tn, rn = clock(lambda: list(pool.map(chunked, chunks)))
        out[name] = {"one_thread": round(nbytes / t1 * 1e-9, 3), "all_threads": round(nbytes / tn * 1e-9, 3)}
        return r1, rn

    with ThreadPoolExecutor(max_workers=threads) as pool:
        amax, parts = both("absmax", 4 * n, lambda: oracle.absmax(v), lambda c: oracle.absmax(v[c[0]:c[1]]), pool)
        assert amax == max(parts)
        for b in (8, 4, 2):
            def quantize_all():
                k, delta, _ = oracle.quantize(v, b, 0, 0, 3)
                return oracle.pack(k, b), delta

            def quantize_chunk(c):
                lo, hi = c
                u = np.concatenate([oracle.uniform_range(0, 0, 3, oracle.TAG_GRAD, lo, hi - lo),
                                    np.array([0.5], dtype=np.float32)])
                k, delta, _ = oracle.quantize_given_uniforms(np.concatenate([v[lo:hi], np.array([amax], dtype=np.float32)]), b, u)
                return oracle.pack(k[:-1], b), delta
            (words, delta), per_chunk = both(f"quantize_pack_b{b}", n * (4 + b / 8), quantize_all, quantize_chunk, pool)
            assert np.array_equal(words, np.concatenate([w for w, _ in per_chunk]))
            rows = np.tile(words, (M, 1))              # M messages (the decode's cost does not depend on their content)
            deltas = np.full(M, delta, dtype=np.float32)
            zeros = np.zeros(n, dtype=np.float32)

            def decode(lo, hi):
                codes = np.stack([oracle.unpack(rows[w, lo * b // 32:hi * b // 32], hi - lo, b) for w in range(M)])
                x = np.zeros(hi - lo, dtype=np.float32)
                # x <- x - eta*(scale*sum_m delta_m k_m + 0) with eta = -1: the aggregated vector itself
                oracle.master_update(codes, deltas, np.float32(1.0 / M), zeros[lo:hi], x, eta=-1.0, l1=0.0)
                return x
            whole, per_chunk = both(f"unpack_dequant_sum_b{b}_M{M}", n * (M * b / 8 + 4), lambda: decode(0, n),
                                    lambda c: decode(c[0], c[1]), pool)
            assert np.array_equal(whole, np.concatenate(per_chunk))
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: the library runs on one GPU (the M workers are a batch dimension on it); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import synth
    import paper_1805_10111_amd as dq
    from paper_1805_10111_amd.driver import DoubleQuantTrainer

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    cfg = synth.CONFIGS[args.config]
    t_gen = time.perf_counter()
    prob = synth.make_problem(cfg, n=args.n)
    t_gen = time.perf_counter() - t_gen
    P = dq.DeviceProblem.from_host(prob)
    tr = DoubleQuantTrainer(P, cfg.algo, cfg.M, cfg.B, cfg.b_x, cfg.b, cfg.m, cfg.lr, seed=cfg.seed)
    tr._t = 0

    m = cfg.m
    meas = time_round_loop(tr, torch, args.steps, args.warmup)
    loop_s, dt, prologue, prologue_s, repeats, wall = (meas[k] for k in ("loop_s", "median_s", "prologue_s", "prologues",
                                                                          "repeats", "wall_s"))

    # ---- dominant kernel: the row-streaming kernel of the worker step (all M workers in one launch), in rounds of
    # its own after the timed region (a launch that carries events is a little slower than one that does not)
    durs = kernel_durations(tr, KERNEL_EPOCHS, EVENT_STRIDE)
    k_avg = float(np.mean(durs))
    if prob.dense is not None:
        rows_bytes = cfg.M * cfg.B * prob.d * 4
    else:
        rows_bytes = int(cfg.M * cfg.B * (prob.indptr[-1] / prob.n) * 8)
    per_worker = tr.xq_words * 4 + prob.d * 4 + tr.row_words * 4 + cfg.B * 8
    alg_bytes = rows_bytes + cfg.M * per_worker
    achieved = alg_bytes / k_avg * 1e-9
    us_round = dt / args.steps * 1e6

    result = {
        "metric": "quantized VR-gradient worker-steps/s + quantize/pack GB/s (% of HBM peak)",
        "value": round(cfg.M * args.steps / dt, 1),
        "unit": "worker-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.algo} logistic, n={prob.n}, d={prob.d}, M={cfg.M}, B={cfg.B}, "
                               f"b_x={cfg.b_x}, b={cfg.b}, m={cfg.m} rounds/epoch, "
                               f"{'CSR' if prob.is_csr else 'dense fp32'}; a step is one round of the inner loop "
                               f"(model message, M worker steps, master step); the epoch prologue (full gradient) "
                               f"is outside the clock and reported in `epoch`",
                   "seed": cfg.seed, "datagen_s": round(t_gen, 1)},
        "timing": {"clock": "HIP events on the launch stream around every run of consecutive rounds of an epoch",
                   "measurement": f"{args.steps} consecutive rounds", "repeats": repeats, "reported": "median",
                   "us_per_round_min_median_max": [round(x / args.steps * 1e6, 2) for x in
                                                   (loop_s[0], dt, loop_s[-1])],
                   "warm_rounds": meas["warm_rounds"],
                   "wall_s_all_repeats_with_prologues": round(wall, 4)},
        "epoch": None if prologue is None else {
            "prologue_us": round(prologue * 1e6, 1), "prologues_timed": len(prologue_s),
            "worker_steps_per_s_with_prologue": round(cfg.M * m / (m * dt / args.steps + prologue), 1),
            "note": "prologue = full gradient at the snapshot (+ the momentum mix of Alg. 3), once per m rounds"},
        "mfma": {"used": False, "why": "the contractions of the path are rows x [d x 2] and [d x rows] x 1: a matrix-core tile "
                                       "would be mostly padding, float32 matrix and vector peaks are equal, and the "
                                       "kernel is bound by the single read of the rows"},
        "roofline": {"bound": "hbm", "kernel": KERNEL_NAME[prob.is_csr],
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": recorded_traffic(cfg.name),
                     "bytes_per_launch": alg_bytes, "avg_launch_us": round(k_avg * 1e6, 2), "launches_timed": len(durs),
                     "timing": f"start/stop HIP events of the kernel's launch, every {EVENT_STRIDE}th round of "
                               f"{KERNEL_EPOCHS} epochs after the timed region",
                     "round_frac": round(alg_bytes / (us_round * 1e-6) * 1e-9 / HBM_PEAK_GBS, 4)},
    }
    del tr, P
    torch.cuda.empty_cache()
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                     # reads 2^30 bytes, writes 2^30 bytes per launch
        torch.cuda.synchronize()
        del src, dst
    if not args.no_other_configs:
        result["other_configs"] = other_configs_leg(dq, torch, synth, DoubleQuantTrainer, args.config)
    if not args.no_quantizer:
        result["quantizer_C5"] = quantizer_leg(dq, torch)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, prob, args.cpu_seconds)
        if not args.no_quantizer:
            result["cpu_baseline"]["quantizer_C5"] = cpu_baseline_quantizer()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
