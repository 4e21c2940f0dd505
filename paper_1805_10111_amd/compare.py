"""Bits-to-loss comparison of the six algorithms of Section 5.1 on a synthetic problem.

AsyLPG, Sparse-AsyLPG, Acc-AsyLPG (double quantization), QSVRG (gradient quantization only) and the
full-precision AsyFPG / Acc-AsyFPG all run through the same kernels (b = 32 / b_x = 32 switch a
quantizer off).  Reports, per algorithm, the objective per epoch and the number of transmitted bits
(worker -> master plus M copies of master -> worker) when the objective at a snapshot first falls below
the threshold, and the saving relative to AsyFPG -- the quantity of Fig. 4 and Table 1 of the paper,
here on synthetic data.

    python -m paper_1805_10111_amd.compare --config C1 --epochs 6 --threshold 0.6

With --mu-sweep it reports instead the study of the precision-loss parameter mu of Section 5.2 (right half of
Table 1): AsyLPG is run once per model width b_x; for each width the run records, round by round, the smallest
mu for which condition (2) holds (E||Q(x)-x||^2 / ||x-x_snap||^2), and the bits transmitted until the
objective falls below the threshold.  A given mu then admits every width whose recorded ratio stays below it.

    python -m paper_1805_10111_amd.compare --config C1 --mu-sweep --widths 2 3 4 5 6 8 10 --epochs 6
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

ALGORITHMS = {                      # name: (loop, b_x, b or None = config's)
    "AsyFPG": ("asylpg", 32, 32),
    "Acc-AsyFPG": ("acc", 32, 32),
    "QSVRG": ("asylpg", 32, None),
    "AsyLPG": ("asylpg", 8, None),
    "Sparse-AsyLPG": ("sparse", 8, None),
    "Acc-AsyLPG": ("acc", 8, None),
}


def run_comparison(cfg, prob, epochs: int, threshold: float, b: int, m: int | None = None, seed: int = 0):
    import paper_1805_10111_amd as dq
    from paper_1805_10111_amd.driver import DoubleQuantTrainer

    P = dq.DeviceProblem.from_host(prob)
    m = cfg.m if m is None else m
    out = {}
    for name, (algo, b_x, bb) in ALGORITHMS.items():
        tr = DoubleQuantTrainer(P, algo, cfg.M, cfg.B, b_x, b if bb is None else bb, m, cfg.lr, seed=seed)
        bits_at, objs, hit = [], [], None
        for e in range(epochs):
            tr.run_epoch()
            objs.append(tr.log.objectives[-1])                 # objective at the start of epoch e
            bits_at.append(tr.log.bits_up + cfg.M * tr.log.bits_down)
        objs.append(tr.objective(tr.x_snap))
        # objective e+1 is reached after the bits of epochs 0..e
        for e in range(epochs):
            if objs[e + 1] < threshold:
                hit = bits_at[e]
                break
        out[name] = {"objectives": [round(o, 6) for o in objs], "bits_total": bits_at[-1], "bits_to_threshold": hit}
    base = out["AsyFPG"]["bits_to_threshold"]
    for name, r in out.items():
        r["saving_vs_AsyFPG"] = None if not (base and r["bits_to_threshold"]) else round(base / r["bits_to_threshold"], 2)
    return out


def mu_sweep(cfg, prob, widths, epochs: int, threshold: float, b: int, m: int | None = None, seed: int = 0,
             mus=(0.005, 0.01, 0.05, 0.1, 0.5, 2.0, 10.0, 50.0, 150.0, 800.0)):
    """Per model width b_x: the mu that condition (2) needs (median and 90th percentile over the rounds after the
    first of each epoch) and the bits to reach the threshold; per mu: the smallest admissible width."""
    import numpy as np
    import paper_1805_10111_amd as dq
    from paper_1805_10111_amd.driver import DoubleQuantTrainer

    P = dq.DeviceProblem.from_host(prob)
    m = cfg.m if m is None else m
    rows = {}
    for b_x in sorted(widths):
        tr = DoubleQuantTrainer(P, "asylpg", cfg.M, cfg.B, b_x, b, m, cfg.lr, seed=seed)
        bits_at, objs, hit = [], [], None
        for e in range(epochs):
            tr.run_epoch(record_mu=True)
            objs.append(tr.log.objectives[-1])
            bits_at.append(tr.log.bits_up + cfg.M * tr.log.bits_down)
        objs.append(tr.objective(tr.x_snap))
        for e in range(epochs):
            if objs[e + 1] < threshold:
                hit = bits_at[e]
                break
        ratios = np.array([err / dist for (_, t, err, dist) in tr.mu_trace if dist > 0.0])
        rows[b_x] = {"mu_needed_median": float(np.median(ratios)), "mu_needed_p90": float(np.quantile(ratios, 0.9)),
                     "final_objective": round(objs[-1], 6), "bits_total": bits_at[-1], "bits_to_threshold": hit}
    choice = {}
    for mu in mus:
        ok = [b_x for b_x in sorted(rows) if rows[b_x]["mu_needed_p90"] <= mu]
        choice[str(mu)] = ok[0] if ok else None
    return {"per_width": rows, "smallest_width_for_mu": choice}


def main():
    import synth
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C1", choices=["C1", "C2", "C4"])
    ap.add_argument("--n", type=int, default=None)
    ap.add_argument("--epochs", type=int, default=6)
    ap.add_argument("--rounds", type=int, default=None, help="rounds per epoch (default: the config's)")
    ap.add_argument("--threshold", type=float, default=0.6)
    ap.add_argument("--bits", type=int, default=8, help="b of the quantized algorithms")
    ap.add_argument("--lr", type=float, default=None, help="step size (default: the config's; the paper tunes it per data set)")
    ap.add_argument("--mu-sweep", action="store_true", help="study of mu / b_x instead of the six-algorithm comparison")
    ap.add_argument("--widths", type=int, nargs="+", default=[2, 3, 4, 5, 6, 7, 8, 9, 10, 11])
    args = ap.parse_args()
    cfg = synth.CONFIGS[args.config]
    if args.lr is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, lr=args.lr)
    prob = synth.make_problem(cfg, n=args.n)
    if args.mu_sweep:
        res = mu_sweep(cfg, prob, args.widths, args.epochs, args.threshold, args.bits, args.rounds)
        print(json.dumps({"config": cfg.name, "n": prob.n, "d": prob.d, "M": cfg.M, "B": cfg.B, "threshold": args.threshold,
                          "b": args.bits, "lr": cfg.lr, "mu_sweep": res}, indent=1))
        return
    res = run_comparison(cfg, prob, args.epochs, args.threshold, args.bits, args.rounds)
    print(json.dumps({"config": cfg.name, "n": prob.n, "d": prob.d, "M": cfg.M, "B": cfg.B, "threshold": args.threshold,
                      "b": args.bits, "lr": cfg.lr, "results": res}, indent=1))


if __name__ == "__main__":
    main()
