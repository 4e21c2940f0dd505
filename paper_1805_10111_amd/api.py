"""ctypes binding of libdq.so: same names and argument order as include/dq.h.

Tensors must live on the GPU (``torch.device('cuda')``) with the dtype the C
signature names; the current PyTorch stream is passed as the HIP stream.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdq.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_DEVICE = 0, -1, -2, -3, -4
TAG_GRAD, TAG_MODEL, TAG_SPARSIFY, TAG_SAMPLE = 0, 1, 2, 3
MASTER_ID = 0xFFFFFFFF
OP_FULL_GRAD, OP_VR_GRAD, OP_WORKER_STEP = 1, 2, 3

_ERR_NAMES = {-1: "DQ_ERR_INVALID_ARG", -2: "DQ_ERR_UNSUPPORTED", -3: "DQ_ERR_WORKSPACE", -4: "DQ_ERR_DEVICE"}


class DqError(RuntimeError):
    def __init__(self, fn: str, code: int, detail: str = ""):
        self.code = code
        super().__init__(f"{fn} returned {_ERR_NAMES.get(code, code)}{detail}")


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_1805_10111_amd/build.py` "
                      "(there is no fallback path)")
_lib = C.CDLL(LIB_PATH)


class _Problem(C.Structure):
    _fields_ = [
        ("layout", C.c_int32),
        ("n", C.c_int64), ("d", C.c_int64),
        ("dense", C.c_void_p), ("lda", C.c_int64),
        ("indptr", C.c_void_p), ("indices", C.c_void_p), ("values", C.c_void_p),
        ("y", C.c_void_p),
        ("l2", C.c_float), ("l1", C.c_float),
    ]


class RunConfig(C.Structure):
    _fields_ = [("algo", C.c_int32), ("M", C.c_int64), ("B", C.c_int64), ("b_x", C.c_int32), ("b", C.c_int32),
                ("m", C.c_int64), ("seed", C.c_uint64), ("tau", C.c_int32), ("each", C.c_int32)]


class RunState(C.Structure):
    _fields_ = [("x", C.c_void_p), ("x_snap", C.c_void_p), ("y", C.c_void_p), ("xsum", C.c_void_p),
                ("g_snap", C.c_void_p), ("z_snap", C.c_void_p), ("xq", C.c_void_p), ("delta_x", C.c_void_p),
                ("absmax_x", C.c_void_p), ("packed", C.c_void_p), ("ld_words", C.c_int64), ("delta", C.c_void_p),
                ("nnz", C.c_void_p), ("status", C.c_void_p), ("ws", C.c_void_p), ("ws_bytes", C.c_int64),
                ("xq_stride_words", C.c_int64), ("wire", C.c_void_p), ("ld_wire", C.c_int64), ("wire_nnz", C.c_void_p)]


ALGO = {"asylpg": 0, "sparse": 1, "acc": 2}

_vp, _i64, _i32, _u64, _u32, _f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_uint32, C.c_float

_SIGS = {
    "dq_version": (C.c_char_p, []),
    "dq_last_device_error": (_i32, []),
    "dq_workspace_bytes": (_i64, [_i32, _vp, _i64, _i64]),
    "dq_workspace_init": (_i32, [_vp, _i64, _vp]),
    "dq_absmax": (_i32, [_vp, _i64, _i64, _i64, _vp, _vp]),
    "dq_quantize": (_i32, [_vp, _i64, _i64, _i64, _i32, _vp, _i32, _u64, _u32, _u32, _u32, _vp, _i64, _vp, _vp, _vp]),
    "dq_dequantize": (_i32, [_vp, _i64, _vp, _i64, _i64, _vp, _i64, _vp]),
    "dq_pack": (_i32, [_vp, _i64, _i64, _i64, _i32, _vp, _i64, _vp]),
    "dq_unpack": (_i32, [_vp, _i64, _i64, _i64, _i32, _vp, _i64, _vp]),
    "dq_quantize_pack": (_i32, [_vp, _i64, _i64, _i64, _i32, _vp, _i32, _u64, _u32, _u32, _u32, _vp, _i64, _vp, _vp, _vp]),
    "dq_unpack_dequant_sum": (_i32, [_vp, _i64, _vp, _i64, _i64, _i32, _f32, _vp, _vp]),
    "dq_sample_indices": (_i32, [_i64, _i64, _i64, _u64, _u32, _u32, _vp, _vp]),
    "dq_full_grad": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _vp]),
    "dq_vr_grad": (_i32, [_vp, _vp, _i64, _i64, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _i64, _vp, _vp, _vp, _i64, _vp]),
    "dq_sparsify": (_i32, [_vp, _i64, _i64, _i64, _vp, _u64, _u32, _u32, _vp, _i64, _vp, _vp, _vp]),
    "dq_worker_step": (_i32, [_vp, _vp, _i64, _i64, _vp, _vp, _i32, _i32, _vp, _vp, _i32, _i32, _u64, _u32, _u32,
                              _vp, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _i64, _vp]),
    "dq_worker_step_static": (_i32, [_vp, _vp, _i64, _i64, _vp, _vp, _i32, _i32, _vp, _vp, _i32, _i32, _u64, _u32, _u32,
                                     _vp, _i64, _vp, _vp, _vp, _i64, _vp, _vp]),
    "dq_master_step": (_i32, [_vp, _i64, _vp, _i64, _i32, _f32, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _i64,
                              _i32, _u64, _u32, _vp, _vp, _vp, _vp, _vp]),
    "dq_master_step_each": (_i32, [_vp, _i64, _vp, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _i64,
                                   _i32, _u64, _u32, _vp, _vp, _vp, _vp, _vp]),
    "dq_acc_params": (_i32, [_f32, _i64, _vp, _vp]),
    "dq_message_bits": (_i64, [_i32, _i64, _i32, _i64]),
    "dq_acc_mix": (_i32, [_vp, _vp, _f32, _i64, _vp, _vp]),
    "dq_acc_snapshot": (_i32, [_vp, _i64, _i64, _vp, _vp]),
    "dq_sparse_stream_words": (_i64, [_i64, _i32]),
    "dq_sparse_encode": (_i32, [_vp, _i64, _i64, _i64, _i32, _vp, _i64, _vp, _vp]),
    "dq_sparse_decode": (_i32, [_vp, _i64, _vp, _i64, _i64, _i32, _vp, _i64, _vp]),
    "dq_mu_terms": (_i32, [_vp, _vp, _i64, _i32, _vp, _vp]),
    "dq_run_rounds": (_i32, [_vp, _vp, _vp, _i64, _i64, _i64, _f32, _f32, _vp, _vp]),
}

EXPORTS = tuple(_SIGS)
_missing = []
for _name, (_res, _args) in _SIGS.items():
    try:
        _f = getattr(_lib, _name)
    except AttributeError:
        _missing.append(_name)
        continue
    _f.restype = _res
    _f.argtypes = _args
if _missing:
    raise ImportError(f"{LIB_PATH} does not export {_missing}: rebuild it")


def _ptr(t: Optional[torch.Tensor], dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor (no CPU path exists)")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(fn: str, rc: int):
    if rc != OK:
        detail = f" (hipError {_lib.dq_last_device_error()})" if rc == ERR_DEVICE else ""
        raise DqError(fn, rc, detail)


def packed_words(d: int, b: int) -> int:
    return (d * b + 31) // 32


def _row_stride(t: torch.Tensor) -> int:
    return t.stride(0) if t.dim() == 2 else t.numel()


def _rows(t: torch.Tensor) -> int:
    return t.shape[0] if t.dim() == 2 else 1


@dataclass
class DeviceProblem:
    """Device-resident problem (eq. (1) with logistic loss); keeps its tensors alive."""

    n: int
    d: int
    y: torch.Tensor
    l2: float
    l1: float
    dense: Optional[torch.Tensor] = None
    indptr: Optional[torch.Tensor] = None
    indices: Optional[torch.Tensor] = None
    values: Optional[torch.Tensor] = None

    def __post_init__(self):
        s = _Problem()
        s.n, s.d = self.n, self.d
        s.y = _ptr(self.y, torch.float32, "y")
        s.l2, s.l1 = self.l2, self.l1
        if self.dense is not None:
            s.layout = 0
            s.dense = _ptr(self.dense, torch.float32, "dense")
            s.lda = self.dense.stride(0)
        else:
            s.layout = 1
            s.indptr = _ptr(self.indptr, torch.int64, "indptr")
            s.indices = _ptr(self.indices, torch.int32, "indices")
            s.values = _ptr(self.values, torch.float32, "values")
        self._s = s

    @property
    def ptr(self):
        return C.addressof(self._s)

    @classmethod
    def from_host(cls, prob, device="cuda") -> "DeviceProblem":
        """Upload a host problem (numpy arrays: see synth.Problem)."""
        t = lambda a: None if a is None else torch.from_numpy(a).to(device)

        def entries(a):                      # a matrix without nonzeros still needs non-null entry arrays
            if a is None:
                return None
            return t(a) if a.size else torch.zeros(1, dtype=torch.from_numpy(a).dtype, device=device)
        return cls(n=prob.n, d=prob.d, y=t(prob.y), l2=float(prob.l2), l1=float(prob.l1), dense=t(prob.dense),
                   indptr=t(prob.indptr), indices=entries(prob.indices), values=entries(prob.values))


# ------------------------------------------------------------------ plumbing
def dq_version() -> str:
    return _lib.dq_version().decode()


def dq_last_device_error() -> int:
    return int(_lib.dq_last_device_error())


def dq_workspace_bytes(op: int, prob: DeviceProblem, M: int, B: int) -> int:
    return int(_lib.dq_workspace_bytes(op, prob.ptr, M, B))


def dq_workspace_init(ws: torch.Tensor) -> None:
    _check("dq_workspace_init", _lib.dq_workspace_init(_ptr(ws, None, "ws"), ws.numel() * ws.element_size(), _stream()))


def new_workspace(op: int, prob: DeviceProblem, M: int = 1, B: int = 1) -> torch.Tensor:
    """Allocates and zero-initialises a workspace for `op` (torch owns the memory)."""
    nbytes = dq_workspace_bytes(op, prob, M, B)
    if nbytes < 0:
        raise DqError("dq_workspace_bytes", nbytes)
    ws = torch.empty((max(nbytes, 16) + 15) // 16 * 4, dtype=torch.float32, device=prob.y.device)
    dq_workspace_init(ws)
    return ws


# ------------------------------------------------------------------ quantizer
def dq_absmax(v: torch.Tensor, absmax_out: torch.Tensor) -> None:
    d, M = v.shape[-1], _rows(v)
    _check("dq_absmax", _lib.dq_absmax(_ptr(v, torch.float32, "v"), d, M, _row_stride(v),
                                       _ptr(absmax_out, torch.float32, "absmax_out"), _stream()))


def dq_quantize(v, b, absmax, absmax_given, seed, it, tag, worker0, codes_out, delta_out, status=None) -> None:
    d, M = v.shape[-1], _rows(v)
    _check("dq_quantize", _lib.dq_quantize(
        _ptr(v, torch.float32, "v"), d, M, _row_stride(v), b, _ptr(absmax, torch.float32, "absmax"), int(absmax_given),
        seed, it, tag, worker0, _ptr(codes_out, torch.int8, "codes_out"), _row_stride(codes_out),
        _ptr(delta_out, torch.float32, "delta_out"), _ptr(status, torch.int32, "status"), _stream()))


def dq_dequantize(codes, delta, d, v_out) -> None:
    M = _rows(codes)
    _check("dq_dequantize", _lib.dq_dequantize(_ptr(codes, torch.int8, "codes"), _row_stride(codes),
                                               _ptr(delta, torch.float32, "delta"), d, M,
                                               _ptr(v_out, torch.float32, "v_out"), _row_stride(v_out), _stream()))


def dq_pack(codes, d, b, packed_out) -> None:
    M = _rows(codes)
    _check("dq_pack", _lib.dq_pack(_ptr(codes, torch.int8, "codes"), _row_stride(codes), d, M, b,
                                   _ptr(packed_out, torch.int32, "packed_out"), _row_stride(packed_out), _stream()))


def dq_unpack(packed, d, b, codes_out) -> None:
    M = _rows(packed)
    _check("dq_unpack", _lib.dq_unpack(_ptr(packed, torch.int32, "packed"), _row_stride(packed), d, M, b,
                                       _ptr(codes_out, torch.int8, "codes_out"), _row_stride(codes_out), _stream()))


def dq_quantize_pack(v, b, absmax, absmax_given, seed, it, tag, worker0, packed_out, delta_out, status=None) -> None:
    d, M = v.shape[-1], _rows(v)
    _check("dq_quantize_pack", _lib.dq_quantize_pack(
        _ptr(v, torch.float32, "v"), d, M, _row_stride(v), b, _ptr(absmax, torch.float32, "absmax"), int(absmax_given),
        seed, it, tag, worker0, _ptr(packed_out, torch.int32, "packed_out"), _row_stride(packed_out),
        _ptr(delta_out, torch.float32, "delta_out"), _ptr(status, torch.int32, "status"), _stream()))


def dq_unpack_dequant_sum(packed, delta, d, b, scale, out) -> None:
    M = _rows(packed)
    _check("dq_unpack_dequant_sum", _lib.dq_unpack_dequant_sum(
        _ptr(packed, torch.int32, "packed"), _row_stride(packed), _ptr(delta, torch.float32, "delta"), d, M, b,
        scale, _ptr(out, torch.float32, "out"), _stream()))


# ------------------------------------------------------------------ sampling, gradients
def dq_sample_indices(n, M, B, seed, it, worker0, idx_out) -> None:
    _check("dq_sample_indices", _lib.dq_sample_indices(n, M, B, seed, it, worker0,
                                                       _ptr(idx_out, torch.int32, "idx_out"), _stream()))


def _ws(ws):
    return (None, 0) if ws is None else (_ptr(ws, None, "ws"), ws.numel() * ws.element_size())


def dq_full_grad(prob: DeviceProblem, x, g_out, z_out=None, obj_out=None, ws=None) -> None:
    wp, wb = _ws(ws)
    _check("dq_full_grad", _lib.dq_full_grad(prob.ptr, _ptr(x, torch.float32, "x"), _ptr(g_out, torch.float32, "g_out"),
                                             _ptr(z_out, torch.float32, "z_out"), _ptr(obj_out, torch.float64, "obj_out"),
                                             wp, wb, _stream()))


def dq_vr_grad(prob: DeviceProblem, idx, M, B, xq_packed, delta_x, b_x, model_is_snapshot, x_snap, z_snap,
               alpha_out, absmax_out, l1norm_out=None, ws=None) -> None:
    wp, wb = _ws(ws)
    _check("dq_vr_grad", _lib.dq_vr_grad(
        prob.ptr, _ptr(idx, torch.int32, "idx"), M, B, _ptr(xq_packed, None, "xq_packed"),
        _ptr(delta_x, torch.float32, "delta_x"), b_x, int(model_is_snapshot), _ptr(x_snap, torch.float32, "x_snap"),
        _ptr(z_snap, torch.float32, "z_snap"), _ptr(alpha_out, torch.float32, "alpha_out"), _row_stride(alpha_out),
        _ptr(absmax_out, torch.float32, "absmax_out"), _ptr(l1norm_out, torch.float32, "l1norm_out"), wp, wb, _stream()))


def dq_sparsify(alpha, phi, seed, it, worker0, beta_out, absmax_out, nnz_out) -> None:
    d, M = alpha.shape[-1], _rows(alpha)
    _check("dq_sparsify", _lib.dq_sparsify(
        _ptr(alpha, torch.float32, "alpha"), d, M, _row_stride(alpha), _ptr(phi, torch.float32, "phi"), seed, it, worker0,
        _ptr(beta_out, torch.float32, "beta_out"), _row_stride(beta_out), _ptr(absmax_out, torch.float32, "absmax_out"),
        _ptr(nnz_out, torch.int32, "nnz_out"), _stream()))


def dq_worker_step(prob: DeviceProblem, idx, M, B, xq_packed, delta_x, b_x, model_is_snapshot, x_snap, z_snap,
                   sparsify, b, seed, it, worker0, packed_out, delta_out, nnz_out=None, alpha_out=None,
                   status=None, ws=None) -> None:
    wp, wb = _ws(ws)
    _check("dq_worker_step", _lib.dq_worker_step(
        prob.ptr, _ptr(idx, torch.int32, "idx"), M, B, _ptr(xq_packed, None, "xq_packed"),
        _ptr(delta_x, torch.float32, "delta_x"), b_x, int(model_is_snapshot), _ptr(x_snap, torch.float32, "x_snap"),
        _ptr(z_snap, torch.float32, "z_snap"), int(sparsify), b, seed, it, worker0,
        _ptr(packed_out, torch.int32, "packed_out"), _row_stride(packed_out), _ptr(delta_out, torch.float32, "delta_out"),
        _ptr(nnz_out, torch.int32, "nnz_out"), _ptr(alpha_out, torch.float32, "alpha_out"),
        0 if alpha_out is None else _row_stride(alpha_out), _ptr(status, torch.int32, "status"), wp, wb, _stream()))


STATIC_WS_BYTES = 8 << 20


def dq_worker_step_static(prob: DeviceProblem, idx, M, B, xq_packed, delta_x, b_x, model_is_snapshot, x_snap, z_snap,
                          sparsify, b, seed, it, worker0, packed_out, delta_out, nnz_out=None, alpha_out=None,
                          status=None) -> None:
    """dq_worker_step on the library's built-in workspace (the call allocates nothing)."""
    _check("dq_worker_step_static", _lib.dq_worker_step_static(
        prob.ptr, _ptr(idx, torch.int32, "idx"), M, B, _ptr(xq_packed, None, "xq_packed"),
        _ptr(delta_x, torch.float32, "delta_x"), b_x, int(model_is_snapshot), _ptr(x_snap, torch.float32, "x_snap"),
        _ptr(z_snap, torch.float32, "z_snap"), int(sparsify), b, seed, it, worker0,
        _ptr(packed_out, torch.int32, "packed_out"), _row_stride(packed_out), _ptr(delta_out, torch.float32, "delta_out"),
        _ptr(nnz_out, torch.int32, "nnz_out"), _ptr(alpha_out, torch.float32, "alpha_out"),
        0 if alpha_out is None else _row_stride(alpha_out), _ptr(status, torch.int32, "status"), _stream()))


# ------------------------------------------------------------------ master
def dq_master_step(packed, delta, M, b, scale, g_snap, x, y, x_snap, xsum, eta, theta, l1, b_x, seed, it,
                   xq_packed_out, delta_x_out, absmax_x_out, status=None) -> None:
    d = x.numel()
    _check("dq_master_step", _lib.dq_master_step(
        _ptr(packed, None, "packed"), _row_stride(packed), _ptr(delta, torch.float32, "delta"), M, b, scale,
        _ptr(g_snap, torch.float32, "g_snap"), _ptr(x, torch.float32, "x"), _ptr(y, torch.float32, "y"),
        _ptr(x_snap, torch.float32, "x_snap"), _ptr(xsum, torch.float32, "xsum"), eta, theta, l1, d, b_x, seed, it,
        _ptr(xq_packed_out, None, "xq_packed_out"), _ptr(delta_x_out, torch.float32, "delta_x_out"),
        _ptr(absmax_x_out, torch.float32, "absmax_x_out"), _ptr(status, torch.int32, "status"), _stream()))


def dq_master_step_each(packed, delta, M, b, g_snap, x, y, x_snap, xsum, eta, theta, l1, b_x, seed, it,
                        xq_packed_out, delta_x_out, absmax_x_out, status=None) -> None:
    d = x.numel()
    _check("dq_master_step_each", _lib.dq_master_step_each(
        _ptr(packed, None, "packed"), _row_stride(packed), _ptr(delta, torch.float32, "delta"), M, b,
        _ptr(g_snap, torch.float32, "g_snap"), _ptr(x, torch.float32, "x"), _ptr(y, torch.float32, "y"),
        _ptr(x_snap, torch.float32, "x_snap"), _ptr(xsum, torch.float32, "xsum"), eta, theta, l1, d, b_x, seed, it,
        _ptr(xq_packed_out, None, "xq_packed_out"), _ptr(delta_x_out, torch.float32, "delta_x_out"),
        _ptr(absmax_x_out, torch.float32, "absmax_x_out"), _ptr(status, torch.int32, "status"), _stream()))


def dq_acc_params(lr: float, s: int):
    """(theta_s, eta_s) of epoch s >= 1 of Alg. 3, as float32 values."""
    theta, eta = C.c_float(), C.c_float()
    _check("dq_acc_params", _lib.dq_acc_params(lr, s, C.byref(theta), C.byref(eta)))
    return theta.value, eta.value


MSG_DENSE, MSG_FLAG, MSG_SPARSE = 0, 1, 2


def dq_message_bits(kind: int, d: int, b: int, nnz: int = 0) -> int:
    bits = int(_lib.dq_message_bits(kind, d, b, nnz))
    if bits < 0:
        raise DqError("dq_message_bits", bits)
    return bits


def dq_acc_mix(y, x_snap, theta, x_out) -> None:
    _check("dq_acc_mix", _lib.dq_acc_mix(_ptr(y, torch.float32, "y"), _ptr(x_snap, torch.float32, "x_snap"), theta,
                                         y.numel(), _ptr(x_out, torch.float32, "x_out"), _stream()))


def dq_acc_snapshot(xsum, m, x_snap_out) -> None:
    _check("dq_acc_snapshot", _lib.dq_acc_snapshot(_ptr(xsum, torch.float32, "xsum"), m, xsum.numel(),
                                                   _ptr(x_snap_out, torch.float32, "x_snap_out"), _stream()))


def dq_sparse_stream_words(d: int, b: int) -> int:
    return int(_lib.dq_sparse_stream_words(d, b))


def dq_sparse_encode(packed, d, b, stream_out, nnz_out) -> None:
    M = _rows(packed)
    _check("dq_sparse_encode", _lib.dq_sparse_encode(_ptr(packed, torch.int32, "packed"), _row_stride(packed), d, M, b,
                                                     _ptr(stream_out, torch.int32, "stream_out"), _row_stride(stream_out),
                                                     _ptr(nnz_out, torch.int32, "nnz_out"), _stream()))


def dq_sparse_decode(stream_in, nnz, d, b, packed_out) -> None:
    M = _rows(stream_in)
    _check("dq_sparse_decode", _lib.dq_sparse_decode(_ptr(stream_in, torch.int32, "stream_in"), _row_stride(stream_in),
                                                     _ptr(nnz, torch.int32, "nnz"), d, M, b,
                                                     _ptr(packed_out, torch.int32, "packed_out"), _row_stride(packed_out),
                                                     _stream()))


def dq_mu_terms(x, x_snap, b, out) -> None:
    _check("dq_mu_terms", _lib.dq_mu_terms(_ptr(x, torch.float32, "x"), _ptr(x_snap, torch.float32, "x_snap"), x.numel(), b,
                                           _ptr(out, torch.float64, "out"), _stream()))


def dq_run_rounds(prob: DeviceProblem, cfg: RunConfig, state: RunState, epoch: int, t0: int, rounds: int,
                  eta: float, theta: float, worker_events=None) -> None:
    """worker_events: optional list of 2*rounds raw hipEvent_t handles (ints; None for a round without events)."""
    ev = None
    if worker_events is not None:
        assert len(worker_events) == 2 * rounds
        ev = (C.c_void_p * len(worker_events))(*worker_events)
    _check("dq_run_rounds", _lib.dq_run_rounds(prob.ptr, C.byref(cfg), C.byref(state), epoch, t0, rounds, eta, theta,
                                               ev, _stream()))


__all__ = [
    "DqError", "DeviceProblem", "EXPORTS", "LIB_PATH", "packed_words",
    "OK", "ERR_INVALID_ARG", "ERR_UNSUPPORTED", "ERR_WORKSPACE", "ERR_DEVICE",
    "TAG_GRAD", "TAG_MODEL", "TAG_SPARSIFY", "TAG_SAMPLE", "MASTER_ID", "OP_FULL_GRAD", "OP_VR_GRAD", "OP_WORKER_STEP",
    "dq_version", "dq_last_device_error", "dq_workspace_bytes", "dq_workspace_init", "new_workspace", "dq_absmax", "dq_quantize", "dq_dequantize",
    "dq_pack", "dq_unpack", "dq_quantize_pack", "dq_unpack_dequant_sum", "dq_sample_indices", "dq_full_grad",
    "dq_vr_grad", "dq_sparsify", "dq_worker_step", "dq_worker_step_static", "STATIC_WS_BYTES", "dq_master_step", "dq_master_step_each", "dq_acc_mix", "dq_acc_snapshot",
    "dq_run_rounds", "dq_mu_terms", "dq_acc_params", "dq_message_bits", "MSG_DENSE", "MSG_FLAG", "MSG_SPARSE", "dq_sparse_stream_words", "dq_sparse_encode", "dq_sparse_decode", "RunConfig", "RunState", "ALGO",
]
