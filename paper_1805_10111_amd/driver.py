"""Epoch loops of AsyLPG / Sparse-AsyLPG / Acc-AsyLPG (Alg. 1-3 of the paper) on one GPU.

Host-side sequencing only: every numerical step is a call into libdq (see include/dq.h).
The M workers of the parameter-server network are one synchronous round: all M read the
same b_x-bit model, the master averages the M decoded b-bit gradients and takes one
proximal (or momentum) step.  ``it = epoch * m + t`` addresses the random streams.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import torch

from . import api as dq


@dataclass
class RunLog:
    objectives: List[float] = field(default_factory=list)   # P(snapshot) at each epoch start, then final
    bits_up: int = 0
    bits_down: int = 0
    rounds: int = 0


class DoubleQuantTrainer:
    """Device-resident state of one run plus the per-epoch call sequence."""

    def __init__(self, prob: dq.DeviceProblem, algo: str, M: int, B: int, b_x: int, b: int, m: int, lr: float,
                 seed: int = 0, x0: Optional[torch.Tensor] = None, cache_margins: bool = True, tau: int = 0,
                 each: bool = False, sparse_wire: bool = False):
        assert algo in ("asylpg", "sparse", "acc")
        self.prob, self.algo, self.M, self.B, self.b_x, self.b, self.m = prob, algo, M, B, b_x, b, m
        self.lr, self.seed, self.tau, self.each = float(lr), int(seed), int(tau), bool(each)
        d, n, dev = prob.d, prob.n, prob.y.device
        f32 = dict(dtype=torch.float32, device=dev)
        i32 = dict(dtype=torch.int32, device=dev)
        self.x_snap = torch.zeros(d, **f32) if x0 is None else x0.to(**f32).clone()
        self.x = self.x_snap.clone()
        self.y = self.x_snap.clone()                   # Alg. 3: y_m^0 = snapshot^0
        self.xsum = torch.zeros(d, **f32)
        self.g_snap = torch.zeros(d, **f32)
        self.z_snap = torch.zeros(n, **f32) if cache_margins else None
        self.obj = torch.zeros(1, dtype=torch.float64, device=dev)
        self.xq_words = d if b_x == 32 else dq.packed_words(d, b_x)
        self.xq_stride = (self.xq_words + 3) // 4 * 4
        self.xq = torch.zeros((self.tau + 1) * self.xq_stride, **i32)     # ring of the last tau+1 model messages
        self.delta_x = torch.zeros(self.tau + 1, **f32)
        self.absmax_x = torch.zeros(2, **f32)
        self.row_words = d if b == 32 else dq.packed_words(d, b)
        self.ld_words = (self.row_words + 3) // 4 * 4
        self.packed = torch.zeros((M, self.ld_words), **i32)
        self.delta = torch.zeros(M, **f32)
        self.nnz = torch.zeros((m, M), **i32)
        self.status = torch.zeros(1, **i32)
        self.ws_full = dq.new_workspace(dq.OP_FULL_GRAD, prob)
        self.ws = dq.new_workspace(dq.OP_VR_GRAD, prob, M, B)
        self.epoch_index = 0
        self.theta, self.eta = 0.0, self.lr
        # Section 4.2 on request (Alg. 2 only): the messages really pass through the sparse (position, value) format
        self.wire = self.wire_nnz = None
        if sparse_wire:
            assert algo == "sparse" and b in (2, 4, 8)
            self.ld_wire = (dq.dq_sparse_stream_words(d, b) + 3) // 4 * 4
            self.wire = torch.zeros((M, self.ld_wire), **i32)
            self.wire_nnz = torch.zeros(M, **i32)
        self.log = RunLog()
        self.mu_trace = []
        p = lambda t: None if t is None else t.data_ptr()
        self.cfg = dq.RunConfig(algo=dq.ALGO[algo], M=M, B=B, b_x=b_x, b=b, m=m, seed=self.seed, tau=self.tau,
                                each=int(self.each))
        self.state = dq.RunState(
            x=p(self.x), x_snap=p(self.x_snap), y=p(self.y), xsum=p(self.xsum), g_snap=p(self.g_snap),
            z_snap=p(self.z_snap), xq=p(self.xq), delta_x=p(self.delta_x), absmax_x=p(self.absmax_x),
            packed=p(self.packed), ld_words=self.ld_words, delta=p(self.delta), nnz=p(self.nnz),
            status=p(self.status), ws=p(self.ws), ws_bytes=self.ws.numel() * 4, xq_stride_words=self.xq_stride,
            wire=p(self.wire), ld_wire=0 if self.wire is None else self.ld_wire, wire_nnz=p(self.wire_nnz))

    # -- one epoch ---------------------------------------------------------------------------
    def epoch_prologue(self) -> None:
        """Epoch start of Alg. 1 / Alg. 3 and the full gradient at the snapshot."""
        e = self.epoch_index
        if self.algo == "acc":
            self.theta, self.eta = dq.dq_acc_params(self.lr, e + 1)        # Section 5.1: theta_s, eta_s
            dq.dq_acc_mix(self.y, self.x_snap, self.theta, self.x)
            self.xsum.zero_()
        else:
            self.theta, self.eta = 0.0, self.lr
            self.x.copy_(self.x_snap)
        dq.dq_full_grad(self.prob, self.x_snap, self.g_snap, self.z_snap, self.obj, self.ws_full)

    def is_flag_round(self, t: int) -> bool:
        """x equals the snapshot bit for bit exactly at the first round of an epoch of Alg. 1/2 and of the
        first epoch of Alg. 3: the master then sends the flag bit of Section 4.1 instead of the model."""
        return t == 0 and (self.algo != "acc" or self.epoch_index == 0)

    def rounds(self, t0: int, count: int, worker_events=None) -> None:
        """Enqueue rounds t0 .. t0+count-1 of the current epoch (one library call).  `worker_events`: optional
        list of 2*count raw hipEvent_t handles recorded around each round's worker-step launches."""
        dq.dq_run_rounds(self.prob, self.cfg, self.state, self.epoch_index, t0, count, self.eta, self.theta,
                         worker_events)

    def round(self, t: int) -> bool:
        self.rounds(t, 1)
        return self.is_flag_round(t)

    def epoch_epilogue(self) -> None:
        if self.algo == "acc":
            dq.dq_acc_snapshot(self.xsum, self.m * (self.M if self.each else 1), self.x_snap)
        else:
            self.x_snap.copy_(self.x)
        self.epoch_index += 1

    def run_epoch(self, record_mu: bool = False) -> None:
        """One epoch.  record_mu: after every round also evaluate both sides of condition (2) for the model
        the master is about to send (appended to ``self.mu_trace`` as [epoch, t, E||Q(x)-x||^2, ||x-x_snap||^2];
        their ratio is the smallest mu for which the condition holds, cf. Fig. 2 of the paper)."""
        self.epoch_prologue()
        if not record_mu or self.b_x == 32:
            self.rounds(0, self.m)
        else:
            buf = torch.zeros((self.m, 2), dtype=torch.float64, device=self.x.device)
            for t in range(self.m):
                self.rounds(t, 1)
                dq.dq_mu_terms(self.x, self.x_snap, self.b_x, buf[t])
            for t, (e, r) in enumerate(buf.cpu().tolist()):
                self.mu_trace.append([self.epoch_index, t, e, r])
        flags = [self.is_flag_round(t) for t in range(self.m)]
        self.epoch_epilogue()
        self._account(flags)

    def _account(self, flags) -> None:
        """Objective at the epoch start and transmitted bits of the epoch (Section 3.1: 32 + b*d bits per
        quantized vector, 32*d unquantized; Section 4.2: position + value per nonzero of a sparsified one)."""
        d, M, m = self.prob.d, self.M, self.m
        self.log.objectives.append(float(self.obj.item()))
        self.log.rounds += m
        for flag in flags:
            self.log.bits_down += dq.dq_message_bits(dq.MSG_FLAG if flag else dq.MSG_DENSE, d, self.b_x)
        if self.algo == "sparse":
            self.log.bits_up += sum(dq.dq_message_bits(dq.MSG_SPARSE, d, self.b, nz)
                                    for nz in self.nnz.flatten().tolist())
        else:
            self.log.bits_up += m * M * dq.dq_message_bits(dq.MSG_DENSE, d, self.b)

    def run(self, S: int) -> RunLog:
        for _ in range(S):
            self.run_epoch()
        self.log.objectives.append(self.objective(self.x_snap))
        if int(self.status.item()) != 0:
            raise FloatingPointError("a quantization scale was not finite (NaN/Inf in a gradient or the model)")
        return self.log

    def objective(self, x: torch.Tensor) -> float:
        g = torch.empty_like(self.g_snap)
        dq.dq_full_grad(self.prob, x, g, None, self.obj, self.ws_full)
        return float(self.obj.item())


def smallest_bx(x: torch.Tensor, x_snap: torch.Tensor, mu: float, candidates=tuple(range(2, 17))) -> int:
    """Smallest b_x among `candidates` for which condition (2) holds with this mu (32 if none does):
    the selection procedure behind the mu / b_x table of Section 5.2."""
    out = torch.zeros((len(candidates), 2), dtype=torch.float64, device=x.device)
    cands = sorted(candidates)
    for i, b in enumerate(cands):
        dq.dq_mu_terms(x, x_snap, b, out[i])
    for b, (e, r) in zip(cands, out.cpu().tolist()):
        if e <= mu * r:
            return b
    return 32
