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
    L.dq_run_rounds.argtypes = [v, v, v, i64, i64, i64, f32, f32, v, v]
    L.dq_acc_params.argtypes = [f32, i64, v, v]
    L.dq_message_bits.restype = C.c_int64
    L.dq_message_bits.argtypes = [i32, i64, i32, i64]
    return L


class RunConfig(C.Structure):
    _fields_ = [("algo", C.c_int32), ("M", C.c_int64), ("B", C.c_int64), ("b_x", C.c_int32), ("b", C.c_int32),
                ("m", C.c_int64), ("seed", C.c_uint64), ("tau", C.c_int32), ("each", C.c_int32)]


class RunState(C.Structure):
    _fields_ = [("x", C.c_void_p), ("x_snap", C.c_void_p), ("y", C.c_void_p), ("xsum", C.c_void_p),
                ("g_snap", C.c_void_p), ("z_snap", C.c_void_p), ("xq", C.c_void_p), ("delta_x", C.c_void_p),
                ("absmax_x", C.c_void_p), ("packed", C.c_void_p), ("ld_words", C.c_int64), ("delta", C.c_void_p),
                ("nnz", C.c_void_p), ("status", C.c_void_p), ("ws", C.c_void_p), ("ws_bytes", C.c_int64),
                ("xq_stride_words", C.c_int64), ("wire", C.c_void_p), ("ld_wire", C.c_int64), ("wire_nnz", C.c_void_p)]


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
    assert full >= 256 * 4096 * 4                      # 256 partial d-vectors at this width (up to 512 at others)
    assert vr >= 32 * 8 * 4096 * 4                     # M * P * d floats with P = 256/M blocks per worker at d = 4096
    # ... and no less than any smaller group of the workers needs (a delayed run steps the groups with this workspace)
    assert all(lib.dq_workspace_bytes(2, C.byref(p), g, 256) <= vr for g in range(1, 33))
    big = dense(d=4096)
    assert all(lib.dq_workspace_bytes(2, C.byref(big), g, 256) <= lib.dq_workspace_bytes(2, C.byref(big), 256, 256)
               for g in (1, 2, 85, 86, 128, 255))
    small = dense(n=2000, d=1000)
    assert lib.dq_workspace_bytes(2, C.byref(small), 4, 16) == 4 * 1 * 1000 * 4       # small batch: one block per worker
    # a row per worker + slice results + one row for (decoded model) - snapshot between the rounds of a call + two sets
    # of prepared mini-batches: per worker 1288 words of row descriptors and a pair of words for each of the
    # (152 KB - 10 KB - 4 * 20960 bytes of LDS) / 12 = 5130 entries that can be staged at this width
    assert lib.dq_workspace_bytes(2, C.byref(csr()), 8, 32) == \
        8 * 20960 * 4 + 8 * 8 * 8 + 20960 * 4 + 2 * 8 * (1288 + 2 * 5130) * 4
    assert lib.dq_workspace_bytes(1, C.byref(csr()), 0, 0) > 256 * 20958 * 4
    # a single step needs none of what dq_run_rounds keeps between the rounds of a call
    assert lib.dq_workspace_bytes(3, C.byref(csr()), 8, 32) == 8 * 20960 * 4 + 8 * 8 * 8
    assert lib.dq_workspace_bytes(3, C.byref(p), 32, 256) == vr
    assert lib.dq_workspace_bytes(4, C.byref(p), 1, 1) == INVALID
    assert lib.dq_workspace_bytes(3, C.byref(p), 0, 256) == INVALID
    assert lib.dq_workspace_bytes(2, C.byref(p), 0, 256) == INVALID
    assert lib.dq_workspace_bytes(1, None, 0, 0) == INVALID


def test_run_rounds_rejects_before_launching(lib):
    """Every rejected call returns before anything is enqueued (the pointers here are never dereferenced)."""
    p = dense()
    ws_need = lib.dq_workspace_bytes(2, C.byref(p), 32, 256)

    def call(tau=0, **over):
        cfg = RunConfig(algo=2, M=32, B=256, b_x=8, b=8, m=25, seed=0, tau=tau, each=0)
        st = RunState(x=P, x_snap=P, y=P, xsum=P, g_snap=P, z_snap=None, xq=P, delta_x=P, absmax_x=P, packed=P,
                      ld_words=1024, delta=P, nnz=None, status=None, ws=P, ws_bytes=ws_need, xq_stride_words=1024)
        for k, val in over.items():
            setattr(st, k, val)
        return lib.dq_run_rounds(C.byref(p), C.byref(cfg), C.byref(st), 0, 0, 1, 0.1, 0.5, None, None)
    assert call(delta_x=None) == INVALID                    # the scale of the model message has nowhere to go
    assert call(tau=2, delta_x=None) == INVALID             # (with a delay, slot arithmetic on a null base is not a pointer)
    assert call(xq=None) == INVALID and call(packed=None) == INVALID and call(y=None) == INVALID
    assert call(status=P + 2) == INVALID and call(nnz=P + 1) == INVALID and call(xq=P + 4) == INVALID
    assert call(ws=None) == WORKSPACE and call(ws_bytes=ws_need - 16) == WORKSPACE
    assert call(tau=2, ws_bytes=32 * 8 * 4096 * 4 - 16) == WORKSPACE     # too small for a group: known up front
    assert call(tau=32) == INVALID


def test_acc_params_and_message_bits(lib):
    import numpy as np
    th, et = C.c_float(), C.c_float()
    for s in (1, 2, 3, 10):
        assert lib.dq_acc_params(0.1, s, C.byref(th), C.byref(et)) == OK
        theta = np.float32(2.0 / (s + 2))                          # Section 5.1
        assert th.value == float(theta) and et.value == float(np.float32(0.1) / theta)
    assert lib.dq_acc_params(0.1, 0, C.byref(th), C.byref(et)) == INVALID
    assert lib.dq_acc_params(0.1, 1, None, C.byref(et)) == INVALID
    bits = lib.dq_message_bits
    assert bits(0, 1000, 8, 0) == 32 + 8 * 1000 and bits(0, 1000, 32, 0) == 32 * 1000        # Section 3.1
    assert bits(0, 20958, 11, 0) == 32 + 11 * 20958
    assert bits(1, 1000, 8, 0) == 1                                                        # Section 4.1
    assert bits(2, 20958, 4, 100) == 32 + 100 * (15 + 4)                                   # Section 4.2: ceil(log2 20958) = 15
    assert bits(2, 4096, 8, 7) == 32 + 7 * (12 + 8) and bits(2, 4097, 8, 7) == 32 + 7 * (13 + 8)
    assert bits(2, 1000, 32, 5) == 5 * (10 + 32)
    assert bits(2, 1000, 4, 1001) == INVALID and bits(3, 1000, 4, 0) == INVALID and bits(0, 1000, 1, 0) == INVALID
    assert bits(0, 0, 8, 0) == INVALID and bits(0, 1000, 17, 0) == INVALID


def test_static_worker_step_rejects_what_does_not_fit(lib):
    lib.dq_worker_step_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32,
                                          C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_uint32,
                                          C.c_uint32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                          C.c_void_p, C.c_void_p]
    wide = dense(n=1000, d=16384)
    assert lib.dq_workspace_bytes(2, C.byref(wide), 64, 256) > 8 << 20
    call = lambda prob, M, B: lib.dq_worker_step_static(C.byref(prob), None, M, B, P, P, 8, 0, P, None, 0, 8, 0, 0, 0, P,
                                                        4096, P, None, None, 0, None, None)
    assert call(wide, 64, 256) == WORKSPACE                 # beyond the built-in workspace: nothing is enqueued
    assert call(dense(), 0, 256) == INVALID


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
