"""Epoch loops of Algorithms 1-3 of the paper, step by step -- TEST INFRASTRUCTURE ONLY.

The M workers of the parameter-server network are taken as one synchronous round:
all M read the same quantized model, the master averages the M decoded gradients and
takes one proximal step (the paper applies gradients one at a time with bounded
staleness; a round with zero staleness is the reading taken here).  The iteration
counter ``it = epoch_index * m + t`` addresses the random streams.

Bounded delay (Assumption 3, Section 3.2) can be emulated: with ``tau > 0`` the M workers are split
into tau+1 contiguous groups and group g computes its gradient on the model message of round
t - g (of round 0 while t < g), i.e. on a model that is g rounds stale.

With ``each=True`` the master follows its rule in Alg. 1 literally: every received gradient triggers
its own update with the full step (the M messages of a round in worker order) instead of one update with
their mean; the model is still sent once per round.  Alg. 3 then averages M*m iterates for the snapshot.

``b_x = 32`` / ``b = 32`` switch the corresponding quantization off (the message is the
float32 vector, 32*d bits): with both off this is AsyFPG / Acc-AsyFPG, with only the model
unquantized it is the gradient-quantized QSVRG arrangement of Section 5.1.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import (MASTER_ID, TAG_GRAD, TAG_MODEL, RefProblem, acc_mix, acc_snapshot, dequantize, dequantize_wide,
               full_grad, master_update, master_update_each, master_update_each_full, master_update_full, objective, pack, pack_wide, quantize, quantize_wide,
               sample_indices, sparsify, unpack, unpack_wide, vr_grad)


@dataclass
class Trace:
    objectives: List[float] = field(default_factory=list)   # P(snapshot) at the start of each epoch, then final
    bits_up: int = 0       # worker -> master
    bits_down: int = 0     # master -> worker (per worker)
    x: Optional[np.ndarray] = None
    x_snap: Optional[np.ndarray] = None


def model_message(x: np.ndarray, x_snap: np.ndarray, b_x: int, seed: int, it: int):
    """Master step (i) of Alg. 1 (model parameter quantization).  Returns (q, packed words or None, delta_x, bits).

    If x equals the snapshot bit for bit the master sends the flag bit of Section 4.1
    and the workers use the snapshot they already hold.
    """
    d = x.size
    if np.array_equal(x.view(np.uint32), x_snap.view(np.uint32)):
        return x_snap.copy(), None, np.float32(0), 1
    if b_x == 32:
        return x.copy(), x.view(np.uint32).copy(), np.float32(1), 32 * d
    if b_x in (2, 4, 8):
        k, dx, _ = quantize(x, b_x, seed, it, MASTER_ID, TAG_MODEL)
        words = pack(k, b_x)
        q = dequantize(unpack(words, d, b_x), dx)
    else:                                            # any other width up to 16 bits (model-precision study, Section 5.2)
        k, dx, _ = quantize_wide(x, b_x, seed, it, MASTER_ID, TAG_MODEL)
        words = pack_wide(k, b_x)
        q = dequantize_wide(unpack_wide(words, d, b_x), dx)
    return q, words, dx, 32 + b_x * d


def worker_message(rp: RefProblem, q, x_snap, model_is_snapshot: bool, B: int, b: int, seed: int,
                   it: int, worker: int, sparse: bool):
    """Worker steps of Alg. 1 ((i), (ii)) and of Alg. 2 ((i)-(iii)).

    Returns (packed words, delta, bits, alpha, beta-or-None, idx).
    """
    d = rp.d
    idx = sample_indices(rp.n, B, seed, it, worker)
    if model_is_snapshot:
        alpha = np.zeros(d, dtype=np.float32)        # grad f_a(xs) - grad f_a(xs)
    else:
        alpha = vr_grad(rp, idx, q, x_snap)
    beta = None
    v = alpha
    nnz = d
    if sparse:
        beta, nnz = sparsify(alpha, seed, it, worker)
        v = beta
    if b == 32:                                      # unquantized message: the vector itself
        nz = int(np.count_nonzero(v))
        bits = 32 * d if not sparse else nz * (math.ceil(math.log2(d)) + 32)
        return v.view(np.uint32).copy(), np.float32(1), bits, alpha, beta, idx
    k, dlt, _ = quantize(v, b, seed, it, worker, TAG_GRAD)
    words = pack(k, b)
    if sparse:
        bits = 32 + int(np.count_nonzero(k)) * (math.ceil(math.log2(d)) + b)
    else:
        bits = 32 + b * d
    return words, dlt, bits, alpha, beta, idx


def worker_delay(w: int, M: int, tau: int) -> int:
    """Staleness (in rounds) of worker w: tau+1 contiguous groups of workers, group g is g rounds behind."""
    return (w * (tau + 1)) // M


def run(prob, algo: str, M: int, B: int, b_x: int, b: int, m: int, S: int, lr: float, seed: int = 0,
        x0: Optional[np.ndarray] = None, eval_objective: bool = True, tau: int = 0, each: bool = False) -> Trace:
    rp = RefProblem(prob)
    d = rp.d
    tr = Trace()
    x_snap = np.zeros(d, dtype=np.float32) if x0 is None else np.array(x0, dtype=np.float32)
    y = x_snap.copy()                     # Acc only: y_m^0 = snapshot^0
    x = x_snap.copy()
    sparse = algo == "sparse"
    for e in range(S):
        if algo == "acc":
            s = e + 1
            theta = np.float32(2.0 / (s + 2))
            eta = np.float32(np.float32(lr) / theta)
            x = acc_mix(y, x_snap, theta)                       # Alg. 3, epoch start
            xsum = np.zeros(d, dtype=np.float32)
        else:
            theta, eta = np.float32(0), np.float32(lr)
            x = x_snap.copy()                                   # Alg. 1, epoch start
        if eval_objective:
            tr.objectives.append(objective(rp, x_snap))
        g_snap = full_grad(rp, x_snap)                          # global gradient   
        history = []                                            # (q, flag) of the model messages of this epoch
        for t in range(m):
            it = e * m + t
            q, _, _, bits = model_message(x, x_snap, b_x, seed, it)
            history.append((q, bits == 1))
            tr.bits_down += bits
            codes = np.zeros((M, d), dtype=np.int8)
            grads = np.zeros((M, d), dtype=np.float32)
            deltas = np.zeros(M, dtype=np.float32)
            for w in range(M):
                q_w, flag_w = history[max(0, t - worker_delay(w, M, tau))]       # x_{D(t)}: a delayed model
                words, dlt, bits, _, _, _ = worker_message(rp, q_w, x_snap, flag_w, B, b, seed, it, w, sparse)
                if b == 32:
                    grads[w] = words.view(np.float32)
                else:
                    codes[w] = unpack(words, d, b)
                deltas[w] = dlt
                tr.bits_up += bits
            yy, ss = (y, xsum) if algo == "acc" else (None, None)     # Alg. 3 / Alg. 1, master (ii)
            if each and b == 32:
                master_update_each_full(grads, g_snap, x, yy, x_snap, ss, eta=eta, theta=theta, l1=rp.l1)
            elif each:
                master_update_each(codes, deltas, g_snap, x, yy, x_snap, ss, eta=eta, theta=theta, l1=rp.l1)
            elif b == 32:
                master_update_full(grads, np.float32(1.0 / M), g_snap, x, yy, x_snap, ss, eta=eta, theta=theta, l1=rp.l1)
            else:
                master_update(codes, deltas, np.float32(1.0 / M), g_snap, x, yy, x_snap, ss, eta=eta, theta=theta,
                              l1=rp.l1)
        if algo == "acc":
            x_snap = acc_snapshot(xsum, m * M if each else m)   # Alg. 3, epoch end: mean of the iterates
        else:
            x_snap = x.copy()                                   # Alg. 1, epoch end
    if eval_objective:
        tr.objectives.append(objective(rp, x_snap))
    tr.x, tr.x_snap = x, x_snap
    return tr
