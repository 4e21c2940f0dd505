"""GPU parity: sparse message encoder/decoder (Section 4.2 of the paper) versus the oracle, bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, words

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1805_10111_amd as dq
    return dq


@pytest.mark.parametrize("b", [2, 4, 8])
@pytest.mark.parametrize("M,d", [(1, 1), (2, 17), (3, 1000), (4, 16385), (16, 20958)])
def test_encode_decode_bit_exact(dq, M, d, b):
    rng = np.random.default_rng(d + b)
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    cap = dq.dq_sparse_stream_words(d, b)
    assert cap == oracle.sparse_stream_words(d, b)
    codes = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d)).astype(np.int8)
    dens = np.linspace(0.0, 1.0, M) if M > 1 else np.array([0.5])
    for m in range(M):
        codes[m, rng.random(d) >= dens[m]] = 0          # from empty to fully dense rows
    pw = np.zeros((M, ldw), dtype=np.uint32)
    for m in range(M):
        pw[m, :nw] = oracle.pack(codes[m], b)
    stream = torch.full((M, cap + 3), -1, dtype=torch.int32, device="cuda")
    nnz = torch.full((M,), -1, dtype=torch.int32, device="cuda")
    dq.dq_sparse_encode(dev(pw.view(np.int32)), d, b, stream, nnz)
    for m in range(M):
        want, k = oracle.sparse_encode(codes[m], b)
        assert host(nnz)[m] == k
        assert np.array_equal(words(stream)[m, :cap], want)
        assert np.all(words(stream)[m, cap:] == 0xFFFFFFFF)
    back = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    dq.dq_sparse_decode(stream, nnz, d, b, back)
    assert np.array_equal(words(back)[:, :nw], pw[:, :nw])


def test_sparse_message_of_a_worker_step(dq):
    """Sparse-AsyLPG message end to end: sparsify -> quantize -> pack -> encode, nnz and bits as in Section 4.2."""
    import synth
    p = synth.sparse_text_logistic(2000, 20958, seed=1)
    P = dq.DeviceProblem.from_host(p)
    M, B, b, d = 4, 16, 4, p.d
    rng = np.random.default_rng(0)
    x_snap = (0.05 * rng.standard_normal(d)).astype(np.float32)
    x = (x_snap + 0.01 * rng.standard_normal(d)).astype(np.float32)
    k, dx, _ = oracle.quantize(x, 8, 1, 1, oracle.MASTER_ID, oracle.TAG_MODEL)
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    packed = torch.zeros((M, ldw), dtype=torch.int32, device="cuda")
    delta = torch.zeros(M, device="cuda")
    nnz = torch.zeros(M, dtype=torch.int32, device="cuda")
    dq.dq_worker_step(P, None, M, B, dev(oracle.pack(k, 8).view(np.int32)), dev(np.array([dx], dtype=np.float32)), 8, False,
                      dev(x_snap), None, True, b, 3, 5, 0, packed, delta, nnz, None, None, None)
    cap = dq.dq_sparse_stream_words(d, b)
    stream = torch.zeros((M, cap), dtype=torch.int32, device="cuda")
    nnz2 = torch.zeros(M, dtype=torch.int32, device="cuda")
    dq.dq_sparse_encode(packed, d, b, stream, nnz2)
    assert torch.equal(nnz, nnz2)
    E = oracle.position_bits(d) + b
    for m in range(M):
        n = int(host(nnz)[m])
        assert 0 < n < d // 4                                         # sparsified: far fewer entries than coordinates
        assert 32 + n * E < 32 + b * d                                 # and a smaller message than the dense one
        used = (n * E + 31) // 32
        assert not words(stream)[m, used:].any()
        codes = oracle.unpack(words(packed)[m, :nw], d, b)
        assert np.array_equal(oracle.sparse_decode(words(stream)[m], n, d, b), codes)


def test_argument_checks(dq):
    p = torch.zeros(64, dtype=torch.int32, device="cuda")
    n = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(dq.DqError) as e:
        dq.dq_sparse_encode(p, 64, 3, p.clone(), n)
    assert e.value.code == dq.ERR_UNSUPPORTED
    with pytest.raises(dq.DqError) as e:                 # stream row shorter than the capacity
        dq.dq_sparse_encode(p, 64, 8, torch.zeros(4, dtype=torch.int32, device="cuda"), n)
    assert e.value.code == dq.ERR_INVALID_ARG
    big = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    with pytest.raises(dq.DqError) as e:                 # stream larger than the on-chip buffer
        dq.dq_sparse_encode(big, 200000, 8, torch.zeros(300000, dtype=torch.int32, device="cuda"), n)
    assert e.value.code == dq.ERR_UNSUPPORTED


@pytest.mark.parametrize("b", [2, 4, 8])
def test_longest_message_the_encoder_takes(dq, b):
    """The encoder assembles a worker's stream in the on-chip buffer (36864 words): the largest d whose full
    stream fits, with one row that has no zero code at all (the stream is at capacity), one empty row and one in
    between; one coordinate more is refused."""
    limit = 36 * 1024
    lo, hi = 1, 1 << 21
    while hi - lo > 1:                                   # largest d with sparse_stream_words(d, b) <= limit
        mid = (lo + hi) // 2
        lo, hi = (mid, hi) if oracle.sparse_stream_words(mid, b) <= limit else (lo, mid)
    d = lo
    assert oracle.sparse_stream_words(d, b) <= limit < oracle.sparse_stream_words(d + 1, b)
    rng = np.random.default_rng(b)
    M = 3
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    cap = dq.dq_sparse_stream_words(d, b)
    codes = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d)).astype(np.int8)
    codes[0][codes[0] == 0] = 1                          # every coordinate present
    codes[1][:] = 0
    codes[2, rng.random(d) < 0.7] = 0
    pw = np.zeros((M, ldw), dtype=np.uint32)
    for m in range(M):
        pw[m, :nw] = oracle.pack(codes[m], b)
    stream = torch.full((M, cap), -1, dtype=torch.int32, device="cuda")
    nnz = torch.full((M,), -1, dtype=torch.int32, device="cuda")
    dq.dq_sparse_encode(dev(pw.view(np.int32)), d, b, stream, nnz)
    for m in range(M):
        want, k = oracle.sparse_encode(codes[m], b)
        assert host(nnz)[m] == k and (m != 0 or k == d)
        assert np.array_equal(words(stream)[m, :cap], want)
    back = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    dq.dq_sparse_decode(stream, nnz, d, b, back)
    assert np.array_equal(words(back)[:, :nw], pw[:, :nw])
    d1 = d + 1
    nw1 = dq.packed_words(d1, b)
    with pytest.raises(dq.DqError) as e:
        dq.dq_sparse_encode(torch.zeros((nw1 + 3) // 4 * 4, dtype=torch.int32, device="cuda"), d1, b,
                            torch.zeros(dq.dq_sparse_stream_words(d1, b), dtype=torch.int32, device="cuda"), nnz[:1])
    assert e.value.code == dq.ERR_UNSUPPORTED
