"""CPU oracle for the double-quantization hot path -- TEST INFRASTRUCTURE ONLY.

ctypes front end of ``dq_oracle.c`` plus the epoch loops of Algorithms 1-3 written
out step by step (``algorithms.py``).  Nothing in the product package imports this;
only tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares no
code with the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dq_oracle.c")
_LIB = os.path.join(_HERE, "libdq_oracle.so")

TAG_GRAD, TAG_MODEL, TAG_SPARSIFY, TAG_SAMPLE = 0, 1, 2, 3
MASTER_ID = 0xFFFFFFFF


def build(force: bool = False) -> str:
    """Compile dq_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _RefProblem(C.Structure):
    _fields_ = [
        ("layout", C.c_int32),
        ("n", C.c_int64), ("d", C.c_int64),
        ("dense", C.c_void_p), ("lda", C.c_int64),
        ("indptr", C.c_void_p), ("indices", C.c_void_p), ("values", C.c_void_p),
        ("y", C.c_void_p),
        ("l2", C.c_float), ("l1", C.c_float),
    ]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ref_random_word.restype = C.c_uint32
        _lib.ref_random_word.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64]
        _lib.ref_uniform.restype = C.c_float
        _lib.ref_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64]
        _lib.ref_uniform_range.restype = None
        _lib.ref_uniform_range.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64, C.c_int64,
                                           C.c_void_p]
        _lib.ref_absmax.restype = C.c_float
        _lib.ref_absmax.argtypes = [C.c_void_p, C.c_int64]
        _lib.ref_delta.restype = C.c_float
        _lib.ref_delta.argtypes = [C.c_float, C.c_int]
        _lib.ref_l1norm.restype = C.c_float
        _lib.ref_l1norm.argtypes = [C.c_void_p, C.c_int64]
        _lib.ref_quantize.restype = C.c_int
        _lib.ref_quantize.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_uint32, C.c_uint32,
                                      C.c_uint32, C.c_void_p, C.c_void_p]
        _lib.ref_quantize_given_uniforms.restype = C.c_int
        _lib.ref_quantize_given_uniforms.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p,
                                                     C.c_void_p]
        _lib.ref_sparsify_given_uniforms.restype = C.c_int64
        _lib.ref_sparsify_given_uniforms.argtypes = [C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p]
        _lib.ref_dequantize.restype = None
        _lib.ref_dequantize.argtypes = [C.c_void_p, C.c_float, C.c_int64, C.c_void_p]
        _lib.ref_packed_words.restype = C.c_int64
        _lib.ref_packed_words.argtypes = [C.c_int64, C.c_int]
        _lib.ref_pack.restype = None
        _lib.ref_pack.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        _lib.ref_unpack.restype = None
        _lib.ref_unpack.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        _lib.ref_quantize_wide.restype = C.c_int
        _lib.ref_quantize_wide.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_uint32, C.c_uint32,
                                           C.c_uint32, C.c_void_p, C.c_void_p]
        _lib.ref_pack_wide.restype = None
        _lib.ref_pack_wide.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        _lib.ref_unpack_wide.restype = None
        _lib.ref_unpack_wide.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        _lib.ref_dequantize_wide.restype = None
        _lib.ref_dequantize_wide.argtypes = [C.c_void_p, C.c_float, C.c_int64, C.c_void_p]
        _lib.ref_master_update_each.restype = None
        _lib.ref_master_update_each.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_float]
        _lib.ref_master_update_each_full.restype = None
        _lib.ref_master_update_each_full.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_float]
        _lib.ref_sample_indices.restype = None
        _lib.ref_sample_indices.argtypes = [C.c_int64, C.c_int64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_void_p]
        _lib.ref_objective.restype = C.c_double
        _lib.ref_objective.argtypes = [C.c_void_p, C.c_void_p]
        _lib.ref_full_grad.restype = None
        _lib.ref_full_grad.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.ref_vr_grad.restype = None
        _lib.ref_vr_grad.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.ref_sparsify.restype = C.c_int64
        _lib.ref_sparsify.argtypes = [C.c_void_p, C.c_int64, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                      C.c_void_p]
        _lib.ref_master_update.restype = None
        _lib.ref_master_update.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_float, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_float, C.c_float, C.c_float]
        _lib.ref_master_update_full.restype = None
        _lib.ref_master_update_full.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_float, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_float, C.c_float, C.c_float]
        _lib.ref_acc_mix.restype = None
        _lib.ref_acc_mix.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int64, C.c_void_p]
        _lib.ref_acc_snapshot.restype = None
        _lib.ref_acc_snapshot.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p]
        _lib.ref_mu_terms.restype = None
        _lib.ref_mu_terms.argtypes = [C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        _lib.ref_expected_sq_error.restype = C.c_double
        _lib.ref_expected_sq_error.argtypes = [C.c_void_p, C.c_int64, C.c_int]
        _lib.ref_sq_distance.restype = C.c_double
        _lib.ref_sq_distance.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        _lib.ref_position_bits.restype = C.c_int
        _lib.ref_position_bits.argtypes = [C.c_int64]
        _lib.ref_sparse_encode.restype = C.c_int64
        _lib.ref_sparse_encode.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_int64]
        _lib.ref_sparse_decode.restype = None
        _lib.ref_sparse_decode.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p]
        _lib.ref_philox4x32_10.restype = None
        _lib.ref_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


# --------------------------------------------------------------------------- RNG
def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().ref_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def random_word(seed: int, it: int, worker: int, tag: int, coord: int) -> int:
    return int(lib().ref_random_word(seed, it, worker, tag, coord))


def uniform(seed: int, it: int, worker: int, tag: int, coord: int) -> float:
    return float(lib().ref_uniform(seed, it, worker, tag, coord))


def uniform_range(seed: int, it: int, worker: int, tag: int, coord0: int, count: int) -> np.ndarray:
    u = np.zeros(count, dtype=np.float32)
    lib().ref_uniform_range(seed, it, worker, tag, coord0, count, _p(u))
    return u


def sample_indices(n: int, B: int, seed: int, it: int, worker: int) -> np.ndarray:
    idx = np.zeros(B, dtype=np.int32)
    lib().ref_sample_indices(n, B, seed, it, worker, _p(idx))
    return idx


# --------------------------------------------------------------------- quantizer
def absmax(v) -> np.float32:
    v = _f32(v)
    return np.float32(lib().ref_absmax(_p(v), v.size))


def delta_of(amax, b: int) -> np.float32:
    return np.float32(lib().ref_delta(np.float32(amax), b))


def l1norm(v) -> np.float32:
    v = _f32(v)
    return np.float32(lib().ref_l1norm(_p(v), v.size))


def quantize(v, b: int, seed: int, it: int, worker: int, tag: int = TAG_GRAD):
    """Returns (codes int8[d], delta float32, status)."""
    v = _f32(v)
    codes = np.zeros(v.size, dtype=np.int8)
    delta = np.zeros(1, dtype=np.float32)
    st = lib().ref_quantize(_p(v), v.size, b, seed, it, worker, tag, _p(codes), _p(delta))
    return codes, delta[0], int(st)


def quantize_given_uniforms(v, b: int, u):
    """Quantizer with the uniform variates supplied by the caller (for exact enumeration)."""
    v, u = _f32(v), _f32(u)
    assert u.size == v.size
    codes = np.zeros(v.size, dtype=np.int8)
    delta = np.zeros(1, dtype=np.float32)
    st = lib().ref_quantize_given_uniforms(_p(v), v.size, b, _p(u), _p(codes), _p(delta))
    return codes, delta[0], int(st)


def dequantize(codes, delta) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    out = np.zeros(codes.size, dtype=np.float32)
    lib().ref_dequantize(_p(codes), np.float32(delta), codes.size, _p(out))
    return out


def packed_words(d: int, b: int) -> int:
    return int(lib().ref_packed_words(d, b))


def pack(codes, b: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    words = np.zeros(packed_words(codes.size, b), dtype=np.uint32)
    lib().ref_pack(_p(codes), codes.size, b, _p(words))
    return words


def unpack(words, d: int, b: int) -> np.ndarray:
    words = np.ascontiguousarray(words, dtype=np.uint32)
    assert words.size >= packed_words(d, b)
    codes = np.zeros(d, dtype=np.int8)
    lib().ref_unpack(_p(words), d, b, _p(codes))
    return codes


# ---- any width 2 <= b <= 16 (int32 codes; fields may straddle words) -------------------
def quantize_wide(v, b: int, seed: int, it: int, worker: int, tag: int = TAG_GRAD):
    """Returns (codes int32[d], delta float32, status) for 2 <= b <= 16."""
    assert 2 <= b <= 16
    v = _f32(v)
    codes = np.zeros(v.size, dtype=np.int32)
    delta = np.zeros(1, dtype=np.float32)
    st = lib().ref_quantize_wide(_p(v), v.size, b, seed, it, worker, tag, _p(codes), _p(delta))
    return codes, delta[0], int(st)


def pack_wide(codes, b: int) -> np.ndarray:
    assert 2 <= b <= 16
    codes = np.ascontiguousarray(codes, dtype=np.int32)
    words = np.zeros(packed_words(codes.size, b), dtype=np.uint32)
    lib().ref_pack_wide(_p(codes), codes.size, b, _p(words))
    return words


def unpack_wide(words, d: int, b: int) -> np.ndarray:
    assert 2 <= b <= 16
    words = np.ascontiguousarray(words, dtype=np.uint32)
    assert words.size >= packed_words(d, b)
    codes = np.zeros(d, dtype=np.int32)
    lib().ref_unpack_wide(_p(words), d, b, _p(codes))
    return codes


def dequantize_wide(codes, delta) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.int32)
    out = np.zeros(codes.size, dtype=np.float32)
    lib().ref_dequantize_wide(_p(codes), np.float32(delta), codes.size, _p(out))
    return out


# ---------------------------------------------------------------------- problem
class RefProblem:
    """Holds host arrays of a synth.Problem alive and exposes the C descriptor."""

    def __init__(self, prob):
        self.n, self.d = prob.n, prob.d
        self.y = _f32(prob.y)
        s = _RefProblem()
        s.n, s.d = prob.n, prob.d
        s.y = _p(self.y)
        s.l2, s.l1 = prob.l2, prob.l1
        if prob.dense is not None:
            self.dense = _f32(prob.dense)
            s.layout, s.dense, s.lda = 0, _p(self.dense), prob.d
        else:
            self.indptr = np.ascontiguousarray(prob.indptr, dtype=np.int64)
            self.indices = np.ascontiguousarray(prob.indices, dtype=np.int32)
            self.values = _f32(prob.values)
            s.layout = 1
            s.indptr, s.indices, s.values = _p(self.indptr), _p(self.indices), _p(self.values)
        self.l2, self.l1 = np.float32(prob.l2), np.float32(prob.l1)
        self._s = s

    @property
    def ptr(self):
        return C.addressof(self._s)


def objective(rp: RefProblem, x) -> float:
    x = _f32(x)
    return float(lib().ref_objective(rp.ptr, _p(x)))


def full_grad(rp: RefProblem, x, want_margins: bool = False):
    x = _f32(x)
    g = np.zeros(rp.d, dtype=np.float32)
    z = np.zeros(rp.n, dtype=np.float32) if want_margins else None
    lib().ref_full_grad(rp.ptr, _p(x), _p(g), _p(z))
    return (g, z) if want_margins else g


def vr_grad(rp: RefProblem, idx, q, x_snap) -> np.ndarray:
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    q, x_snap = _f32(q), _f32(x_snap)
    a = np.zeros(rp.d, dtype=np.float32)
    lib().ref_vr_grad(rp.ptr, _p(idx), idx.size, _p(q), _p(x_snap), _p(a))
    return a


def sparsify(alpha, seed: int, it: int, worker: int, phi: float = -1.0):
    """Returns (beta float32[d], nnz).  phi < 0: the budget ||alpha||_1/||alpha||_inf."""
    alpha = _f32(alpha)
    beta = np.zeros(alpha.size, dtype=np.float32)
    nnz = lib().ref_sparsify(_p(alpha), alpha.size, np.float32(phi), seed, it, worker, _p(beta))
    return beta, int(nnz)


def sparsify_given_uniforms(alpha, u, phi: float = -1.0):
    alpha, u = _f32(alpha), _f32(u)
    assert u.size == alpha.size
    beta = np.zeros(alpha.size, dtype=np.float32)
    nnz = lib().ref_sparsify_given_uniforms(_p(alpha), alpha.size, np.float32(phi), _p(u), _p(beta))
    return beta, int(nnz)


def master_update(codes, delta, scale, g_snap, x, y=None, x_snap=None, xsum=None,
                  eta=0.0, theta=0.0, l1=0.0) -> None:
    """In-place update of x (and y, xsum).  codes: int8 [M, d]; delta: float32 [M]."""
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    delta = _f32(delta)
    M, d = codes.shape
    for a in (g_snap, x, y, x_snap, xsum):
        assert a is None or (a.dtype == np.float32 and a.flags.c_contiguous and a.size == d)
    lib().ref_master_update(_p(codes), _p(delta), M, d, np.float32(scale), _p(g_snap), _p(x), _p(y),
                            _p(x_snap), _p(xsum), np.float32(eta), np.float32(theta), np.float32(l1))


def master_update_full(grads, scale, g_snap, x, y=None, x_snap=None, xsum=None, eta=0.0, theta=0.0, l1=0.0) -> None:
    """Master update from unquantized gradients: grads float32 [M, d]."""
    grads = np.ascontiguousarray(grads, dtype=np.float32)
    M, d = grads.shape
    for a in (g_snap, x, y, x_snap, xsum):
        assert a is None or (a.dtype == np.float32 and a.flags.c_contiguous and a.size == d)
    lib().ref_master_update_full(_p(grads), M, d, np.float32(scale), _p(g_snap), _p(x), _p(y), _p(x_snap),
                                 _p(xsum), np.float32(eta), np.float32(theta), np.float32(l1))


def master_update_each(codes, delta, g_snap, x, y=None, x_snap=None, xsum=None, eta=0.0, theta=0.0, l1=0.0) -> None:
    """One master update per received gradient (the M messages of a round in worker order); in place."""
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    M, d = codes.shape
    delta = _f32(delta)
    assert delta.size == M
    for a in (g_snap, x, y, x_snap, xsum):
        assert a is None or (a.dtype == np.float32 and a.flags.c_contiguous and a.size == d)
    lib().ref_master_update_each(_p(codes), _p(delta), M, d, _p(g_snap), _p(x), _p(y), _p(x_snap), _p(xsum),
                                 np.float32(eta), np.float32(theta), np.float32(l1))


def master_update_each_full(grads, g_snap, x, y=None, x_snap=None, xsum=None, eta=0.0, theta=0.0, l1=0.0) -> None:
    grads = np.ascontiguousarray(grads, dtype=np.float32)
    M, d = grads.shape
    for a in (g_snap, x, y, x_snap, xsum):
        assert a is None or (a.dtype == np.float32 and a.flags.c_contiguous and a.size == d)
    lib().ref_master_update_each_full(_p(grads), M, d, _p(g_snap), _p(x), _p(y), _p(x_snap), _p(xsum),
                                      np.float32(eta), np.float32(theta), np.float32(l1))


def acc_mix(y, x_snap, theta) -> np.ndarray:
    y, x_snap = _f32(y), _f32(x_snap)
    out = np.zeros_like(y)
    lib().ref_acc_mix(_p(y), _p(x_snap), np.float32(theta), y.size, _p(out))
    return out


def acc_snapshot(xsum, m: int) -> np.ndarray:
    xsum = _f32(xsum)
    out = np.zeros_like(xsum)
    lib().ref_acc_snapshot(_p(xsum), m, xsum.size, _p(out))
    return out


def mu_terms(codes, delta, x, x_snap):
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    x, x_snap = _f32(x), _f32(x_snap)
    out = np.zeros(2, dtype=np.float64)
    lib().ref_mu_terms(_p(codes), np.float32(delta), _p(x), _p(x_snap), x.size, _p(out))
    return out


def expected_sq_error(x, b: int) -> float:
    """E_Q ||Q(x) - x||^2 for the b-bit quantizer with the max-norm scale (left side of condition (2))."""
    x = _f32(x)
    return float(lib().ref_expected_sq_error(_p(x), x.size, b))


def sq_distance(x, x_snap) -> float:
    x, x_snap = _f32(x), _f32(x_snap)
    return float(lib().ref_sq_distance(_p(x), _p(x_snap), x.size))


def smallest_bx(x, x_snap, mu: float, candidates=tuple(range(2, 17))) -> int:
    """Smallest b_x among `candidates` that satisfies condition (2) for this mu; 32 if none does."""
    r = sq_distance(x, x_snap)
    for b in sorted(candidates):
        if expected_sq_error(x, b) <= mu * r:
            return b
    return 32


def position_bits(d: int) -> int:
    return int(lib().ref_position_bits(d))


def sparse_stream_words(d: int, b: int) -> int:
    """Words that hold the sparse message when every coordinate is nonzero."""
    return (d * (position_bits(d) + b) + 31) // 32


def sparse_encode(codes, b: int):
    """Returns (stream words uint32[capacity], nnz): position+value per nonzero code (Section 4.2)."""
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    cap = sparse_stream_words(codes.size, b)
    words = np.zeros(cap, dtype=np.uint32)
    nnz = lib().ref_sparse_encode(_p(codes), codes.size, b, _p(words), cap)
    return words, int(nnz)


def sparse_decode(words, nnz: int, d: int, b: int) -> np.ndarray:
    words = np.ascontiguousarray(words, dtype=np.uint32)
    codes = np.zeros(d, dtype=np.int8)
    lib().ref_sparse_decode(_p(words), nnz, d, b, _p(codes))
    return codes
