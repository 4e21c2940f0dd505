"""Host-side logic of the C ABI that runs before any GPU work: argument validation and workspace sizes.

Pointers handed over here are never dereferenced (every call below is rejected, or is pure host
arithmetic), so the tests run without a GPU.
"""
import ctypes as C
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1805_10111_amd", "libdq.so")

OK, INVALID, UNSUPPORTED, WORKSPACE = 0, -1, -2, -3
P = 0x10000          # a 16-byte aligned, never dereferenced "device pointer"


class Problem(C.Structure):
    _fields_ = [("layout", C.c_int32), ("n", C.c_int64), ("d", C.c_int64), ("dense", C.c_void_p), ("lda", C.c_int64),
                ("indptr", C.c_void_p), ("indices", C.c_void_p), ("values", C.c_void_p), ("y", C.c_void_p),
                ("l2", C.c_float), ("l1", C.c_float)]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} not built: run python paper_1805_10111_amd/build.py")
    L = C.CDLL(LIB)
    L.dq_workspace_bytes.restype = C.c_int64
    L.dq_workspace_bytes.argtypes = [C.c_int32, C.c_void_p, C.c_int64, C.c_int64]
    v, i64, i32, u64, u32, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_uint32, C.c_float
    L.dq_quantize_pack.argtypes = [v, i64, i64, i64, i32, v, i32, u64, u32, u32, u32, v, i64, v, v, v]
    L.dq_quantize.argtypes = [v, i64, i64, i64, i32, v, i32, u64, u32, u32, u32, v, i64, v, v, v]
    L.dq_pack.argtypes = [v, i64, i64, i64, i32, v, i64, v]
    L.dq_unpack_dequant_sum.argtypes = [v, i64, v, i64, i64, i32, f32, v, v]
    L.dq_absmax.argtypes = [v, i64, i64, i64, v, v]
    L.dq_master_step.argtypes = [v, i64, v, i64, i32, f32, v, v, v, v, v, f32, f32, f32, i64, i32, u64, u32, v, v, v, v, v]
    L.dq_full_grad.argtypes = [v, v, v, v, v, v, i64, v]
    L.dq_sample_indices.argtypes = [i64, i64, i64, u64, u32, u32, v, v]
    L.dq_worker_step.argtypes = [v, v, i64, i64, v, v, i32, i32, v, v, i32, i32, u64, u32, u32, v, i64, v, v, v, i64, v,
                                 v, i64, v]
    return L


def dense(n=200000, d=4096, lda=None):
    return Problem(layout=0, n=n, d=d, dense=P, lda=d if lda is None else lda, y=P)


def csr(n=72000, d=20958):
    return Problem(layout=1, n=n, d=d, indptr=P, indices=P, values=P, y=P)


def test_quantizer_argument_checks(lib):
    q = lambda b, v=P, d=64, M=1, ld=64, out=P, ldw=16: lib.dq_quantize_pack(v, d, M, ld, b, P, 0, 0, 0, 0, 0, out, ldw, P, None, None)
    assert q(1) == INVALID and q(0) == INVALID and q(17) == INVALID and q(33) == INVALID      # widths 2..16 only
    assert q(8, v=None) == INVALID and q(8, out=None) == INVALID
    assert q(8, v=P + 4) == INVALID                                  # misaligned
    assert q(8, d=-1) == INVALID and q(8, M=0) == INVALID
    assert q(8, M=2, ld=63) == INVALID                               # stride shorter than the row
    assert q(8, M=2, ld=66) == INVALID                               # stride not a multiple of 4
    assert q(8, d=64, ldw=15) == INVALID                             # packed row too short
    assert lib.dq_quantize(P, 64, 1, 64, 8, P, 0, 0, 0, 0, 0, P, 62, P, None, None) == INVALID
    assert lib.dq_pack(P, 64, 64, 1, 9, P, 16, None) == INVALID                         # int8 codes: at most 8 bits
    assert lib.dq_pack(P, 64, 64, 1, 1, P, 16, None) == INVALID
    assert lib.dq_unpack_dequant_sum(P, 16, None, 64, 1, 8, 1.0, P, None) == INVALID     # no delta
    assert lib.dq_unpack_dequant_sum(P, 16, P, 64, 1, 17, 1.0, P, None) == INVALID
    assert lib.dq_absmax(P, 64, 1, 64, None, None) == INVALID
    assert lib.dq_sample_indices(0, 1, 1, 0, 0, 0, P, None) == INVALID
    assert lib.dq_sample_indices(2**31, 1, 1, 0, 0, 0, P, None) == INVALID


def test_master_argument_checks(lib):
    m = lambda b=8, bx=8, y=None, xs=P, d=64, ldw=16, delta=P: lib.dq_master_step(
        P, ldw, delta, 2, b, 0.5, P, P, y, xs, None, 0.1, 0.5, 0.0, d, bx, 0, 0, P, P, P, None, None)
    assert m(b=3) == UNSUPPORTED                                     # gradient messages: 2, 4, 8 or 32 bits
    assert m(b=1) == INVALID and m(bx=64) == INVALID and m(bx=17) == INVALID and m(bx=1) == INVALID
    assert m(y=P, xs=None) == INVALID                                # momentum update without a snapshot
    assert m(d=0) == INVALID and m(ldw=3) == INVALID and m(delta=None) == INVALID
    assert m(ldw=18) == INVALID                                      # M > 1 rows must keep 16-byte alignment


def test_problem_and_gradient_argument_checks(lib):
    p = dense()
    assert lib.dq_full_grad(C.byref(p), P, P, None, None, None, 0, None) == WORKSPACE
    assert lib.dq_full_grad(C.byref(p), None, P, None, None, P, 1 << 40, None) == INVALID
    bad = dense(lda=4095)
    assert lib.dq_full_grad(C.byref(bad), P, P, None, None, P, 1 << 40, None) == INVALID
    wide = dense(d=20000, lda=20000)               # dense rows of more than 16384 floats
    assert lib.dq_full_grad(C.byref(wide), P, P, None, None, P, 1 << 40, None) == UNSUPPORTED
    huge = csr(d=1 << 20)                          # staged entries address fewer than 2^20 columns
    assert lib.dq_full_grad(C.byref(huge), P, P, None, None, P, 1 << 40, None) == UNSUPPORTED
    none = Problem(layout=2, n=1, d=1, y=P)
    assert lib.dq_full_grad(C.byref(none), P, P, None, None, P, 1 << 40, None) == INVALID
    w = lambda prob, b=8, bx=8, ldw=1024, ws=P, wsb=1 << 40, idx=None, xq=P: lib.dq_worker_step(
        C.byref(prob), idx, 32, 256, xq, P, bx, 0, P, None, 0, b, 0, 0, 0, P, ldw, P, None, None, 0, None, ws, wsb, None)
    assert w(p, b=3) == UNSUPPORTED and w(p, b=16) == INVALID and w(p, bx=17) == INVALID and w(p, bx=1) == INVALID
    assert w(p, ldw=1023) == INVALID and w(p, xq=None) == INVALID
    assert w(p, ws=None, wsb=0) == WORKSPACE and w(p, wsb=1024) == WORKSPACE


def test_workspace_sizes(lib):
    p = dense()
    full = lib.dq_workspace_bytes(1, C.byref(p), 0, 0)
    vr = lib.dq_workspace_bytes(2, C.byref(p), 32, 256)
    assert full % 16 == 0 and vr % 16 == 0
    assert full >= 512 * 4096 * 4                      # up to 512 partial d-vectors
    assert vr == 32 * 8 * 4096 * 4                     # M * P * d floats with P = 256/M blocks per worker at d = 4096
    small = dense(n=2000, d=1000)
    assert lib.dq_workspace_bytes(2, C.byref(small), 4, 16) == 4 * 1 * 1000 * 4       # small batch: one block per worker
    assert lib.dq_workspace_bytes(2, C.byref(csr()), 8, 32) == 8 * 20960 * 4 + 8 * 8 * 8   # a row per worker + slice results
    assert lib.dq_workspace_bytes(1, C.byref(csr()), 0, 0) > 256 * 20958 * 4
    assert lib.dq_workspace_bytes(3, C.byref(p), 1, 1) == INVALID
    assert lib.dq_workspace_bytes(2, C.byref(p), 0, 256) == INVALID
    assert lib.dq_workspace_bytes(1, None, 0, 0) == INVALID


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
