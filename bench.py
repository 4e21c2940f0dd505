#!/usr/bin/env python3
"""Benchmark of the double-quantization hot path on one MI355X.

A step is one synchronous round of the whole path for all M workers: model message ->
variance-reduced mini-batch gradients -> stochastic quantization -> packing -> master
decode/aggregate -> prox or momentum update -> model re-quantization, with the epoch
prologue (full gradient) executed inside the timed region at its real cadence (every m
rounds).  Inputs are resident in HBM before the clock starts.

Prints ONE JSON line: worker-steps/s (= M * rounds / time) on the accelerated dense
workload (config C4), the roofline figures of the dominant kernel measured with HIP
events on the launch stream, the quantizer microbenchmark (config C5) as extra fields,
and the CPU oracle timed on a bounded sample of the same workload.
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
EVENT_STRIDE = 8          # rounds between HIP-event brackets around the dominant kernel
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


def run_rounds(tr, rounds, events=None):
    """Advance the trainer by `rounds` rounds, running epoch prologues/epilogues at their cadence.

    `events`: optional list that receives (start, end, is_flag_round) for the bracketed rounds, the two
    torch events being handed to the library as the start and stop events of the launch of the kernel that
    streams the feature rows (the dominant kernel of a round).
    """
    import torch
    done = 0
    while done < rounds:
        if tr._t == 0:
            tr.epoch_prologue()
        take = min(rounds - done, tr.m - tr._t)
        if events is None:
            tr.rounds(tr._t, take)
        else:
            # only every EVENT_STRIDE-th round is bracketed (a launch that carries events is a little slower)
            k = 0
            while k < take:
                if (done + k) % EVENT_STRIDE == EVENT_STRIDE - 1:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(); e1.record()            # instantiates the HIP events; the launch overwrites them
                    tr.rounds(tr._t + k, 1, [e0.cuda_event, e1.cuda_event])
                    events.append((e0, e1, tr.is_flag_round(tr._t + k)))
                    k += 1
                else:
                    run = min(take - k, EVENT_STRIDE - 1 - (done + k) % EVENT_STRIDE)
                    tr.rounds(tr._t + k, run)
                    k += run
        tr._t += take
        done += take
        if tr._t == tr.m:
            tr.epoch_epilogue()
            tr._t = 0


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
        run_rounds(tr, cfg.m)                      # one epoch of warm-up
        torch.cuda.synchronize()
        rounds = 2 * cfg.m
        t0 = time.perf_counter()
        run_rounds(tr, rounds)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        out[name] = {"us_per_round": round(dt / rounds * 1e6, 2), "worker_steps_per_s": round(cfg.M * rounds / dt, 1),
                     "rounds": rounds, "M": cfg.M, "B": cfg.B, "d": prob.d,
                     "note": "launch/latency-bound: under 3 MB of traffic per round"}
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

    run_rounds(tr, args.warmup)
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    run_rounds(tr, args.steps, events)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if int(tr.status.item()) != 0:
        raise FloatingPointError("non-finite quantization scale during the benchmark")

    # the same rounds without the epoch prologue (rate of the inner loop alone): whole epochs, prologue outside
    # the clock, no event brackets
    while tr._t != 0:
        run_rounds(tr, 1)
    inner_s, inner_rounds = 0.0, 0
    for _ in range(max(1, min(8, args.steps // cfg.m))):
        tr.epoch_prologue()
        torch.cuda.synchronize()
        ti = time.perf_counter()
        tr.rounds(0, tr.m)
        torch.cuda.synchronize()
        inner_s += time.perf_counter() - ti
        inner_rounds += tr.m
        tr.epoch_epilogue()

    # dominant kernel: the row-streaming kernel of the worker step (all M workers in one launch);
    # flag-bit rounds read no rows and are skipped.  The two events are the start and stop events of that launch
    # (hipExtLaunchKernel inside the library), i.e. the kernel's own duration on the launch stream.
    durs = [e0.elapsed_time(e1) * 1e-3 for e0, e1, flag in events if not flag]
    k_avg = float(np.mean(durs))
    if prob.dense is not None:
        rows_bytes = cfg.M * cfg.B * prob.d * 4
    else:
        rows_bytes = int(cfg.M * cfg.B * (prob.indptr[-1] / prob.n) * 8)
    per_worker = tr.xq_words * 4 + prob.d * 4 + tr.row_words * 4 + cfg.B * 8
    alg_bytes = rows_bytes + cfg.M * per_worker
    achieved = alg_bytes / k_avg * 1e-9

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
                               f"{'CSR' if prob.is_csr else 'dense fp32'}; full gradient every m rounds inside the timed region",
                   "seed": cfg.seed, "datagen_s": round(t_gen, 1),
                   "inner_loop_only": {"worker_steps_per_s": round(cfg.M * inner_rounds / inner_s, 1),
                                       "us_per_round": round(inner_s / inner_rounds * 1e6, 2),
                                       "note": "rounds of whole epochs with the full gradient outside the clock"}},
        "mfma": {"used": False, "why": "the contractions of the path are rows x [d x 2] and [d x rows] x 1: a matrix-core tile "
                                       "would be mostly padding, float32 matrix and vector peaks are equal, and the "
                                       "kernel is bound by the single read of the rows"},
        "roofline": {"bound": "hbm", "kernel": KERNEL_NAME[prob.is_csr],
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": recorded_traffic(cfg.name),
                     "bytes_per_launch": alg_bytes, "avg_launch_us": round(k_avg * 1e6, 2),
                     "timing": "start/stop HIP events of the kernel's launch, every 8th round of the timed region"},
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
    print(json.dumps(result))


if __name__ == "__main__":
    main()
