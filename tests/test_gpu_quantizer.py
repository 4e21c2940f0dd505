"""GPU parity: quantizer family through the C ABI versus the CPU oracle (bit-exact)."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import dev, host, words

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1805_10111_amd as dq
    return dq


# sizes: empty-ish, sub-chunk, ragged tails around 16 / 4096, several blocks
SIZES = [1, 3, 15, 16, 17, 250, 1000, 4096, 4097, 20958, 70001]


def _vec(d, seed):
    return synth.mixture_vector(d, seed=seed)


@pytest.mark.parametrize("d", SIZES)
def test_absmax(dq, d):
    v = _vec(d, d)
    out = torch.full((1,), -1.0, device="cuda")
    dq.dq_absmax(dev(v), out)
    assert host(out)[0] == oracle.absmax(v)


def test_absmax_rows_and_nan(dq):
    M, d, ld = 5, 1001, 1004
    buf = np.zeros((M, ld), dtype=np.float32)
    rng = np.random.default_rng(0)
    buf[:, :d] = rng.standard_normal((M, d)).astype(np.float32)
    buf[:, d:] = 1e9            # padding must be ignored
    buf[3, 17] = np.nan
    t = dev(buf)[:, :d]
    out = torch.zeros(M, device="cuda")
    dq.dq_absmax(t, out)
    got = host(out)
    for m in range(M):
        want = oracle.absmax(buf[m, :d])
        assert (np.isnan(got[m]) and np.isnan(want)) or got[m] == want


@pytest.mark.parametrize("b", [2, 4, 8])
@pytest.mark.parametrize("d", SIZES)
def test_quantize_pack_bit_exact(dq, d, b):
    v = _vec(d, 100 + d)
    seed, it, worker = 0x1234567890ABCDEF, 7, 3
    nw = dq.packed_words(d, b)
    packed = torch.full((nw + 4,), -1, dtype=torch.int32, device="cuda")
    absmax = torch.zeros(1, device="cuda")
    delta = torch.zeros(1, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    dq.dq_quantize_pack(dev(v), b, absmax, False, seed, it, dq.TAG_GRAD, worker, packed, delta, status)
    k, dlt, st = oracle.quantize(v, b, seed, it, worker, oracle.TAG_GRAD)
    assert host(delta)[0] == dlt and host(absmax)[0] == oracle.absmax(v)
    assert host(status)[0] == st == 0
    assert np.array_equal(words(packed)[:nw], oracle.pack(k, b))
    assert np.all(words(packed)[nw:] == 0xFFFFFFFF)          # nothing written past the row


@pytest.mark.parametrize("b", [2, 3, 5, 8])
def test_quantize_int8_codes_rows(dq, b):
    M, d, ld = 4, 1003, 1008
    rng = np.random.default_rng(b)
    buf = rng.standard_normal((M, ld)).astype(np.float32)
    v = dev(buf)[:, :d]
    codes = torch.zeros((M, 1008), dtype=torch.int8, device="cuda")[:, :d]
    absmax = torch.zeros(M, device="cuda")
    delta = torch.zeros(M, device="cuda")
    dq.dq_quantize(v, b, absmax, False, 5, 2, dq.TAG_MODEL, 10, codes, delta)
    back = torch.zeros((M, ld), device="cuda")[:, :d]
    dq.dq_dequantize(codes, delta, d, back)
    for m in range(M):
        k, dlt, _ = oracle.quantize(buf[m, :d], b, 5, 2, 10 + m, oracle.TAG_MODEL)
        assert host(delta)[m] == dlt
        assert np.array_equal(host(codes)[m], k)
        assert np.array_equal(host(back)[m], oracle.dequantize(k, dlt))


def test_absmax_given_is_used(dq):
    d = 500
    v = _vec(d, 1)
    amax = np.float32(2.0) * oracle.absmax(v)          # caller's (larger) scale numerator
    absmax = dev(np.array([amax], dtype=np.float32))
    codes = torch.zeros(512, dtype=torch.int8, device="cuda")[:d]
    delta = torch.zeros(1, device="cuda")
    dq.dq_quantize(dev(v), 8, absmax, True, 1, 1, dq.TAG_GRAD, 0, codes, delta)
    assert host(delta)[0] == oracle.delta_of(amax, 8)
    assert np.abs(host(codes)).max() <= 64


@pytest.mark.parametrize("b", [2, 4, 8])
def test_scale_smaller_than_the_vector_clamps_like_the_rule(dq, b):
    """A caller-supplied ||v||_inf below the true maximum (outside the paper's definition, which always takes the
    true one): values beyond the scale get the end codes of the b-bit range, -2^(b-1) and 2^(b-1)-1, and all others
    the code of the rule of Section 3.1 with the stream's uniform variates.  The expected codes apply that rule in
    float32 with the oracle's variates; the oracle's own quantizer always derives the scale from the vector."""
    d = 4099
    v = _vec(d, 3)
    amax = np.float32(0.05) * oracle.absmax(v)
    L = np.float32(2 ** (b - 1) - 1)
    inv_delta = L / amax
    t = (v * inv_delta).astype(np.float32)
    z = np.floor(t)
    p = (t - z).astype(np.float32)
    u = oracle.uniform_range(9, 4, 2, oracle.TAG_GRAD, 0, d)
    want = np.clip(z.astype(np.int64) + (u < p), -(2 ** (b - 1)), 2 ** (b - 1) - 1)
    assert (np.abs(t) > L + 2).sum() > 50                     # the case is really exercised
    codes = torch.zeros((1, 4112), dtype=torch.int8, device="cuda")[:, :d]
    delta = torch.zeros(1, device="cuda")
    dq.dq_quantize(dev(v)[None, :], b, dev(np.array([amax], dtype=np.float32)), True, 9, 4, dq.TAG_GRAD, 2, codes, delta)
    assert np.array_equal(host(codes)[0].astype(np.int64), want)
    assert host(delta)[0] == oracle.delta_of(amax, b)


@pytest.mark.parametrize("b", [2, 4, 8])
def test_pack_unpack_roundtrip(dq, b):
    M, d = 3, 1001
    rng = np.random.default_rng(b)
    k = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d)).astype(np.int8)
    kbuf = np.zeros((M, 1008), dtype=np.int8)
    kbuf[:, :d] = k
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    packed = torch.full((M, ldw), -1, dtype=torch.int32, device="cuda")
    dq.dq_pack(dev(kbuf)[:, :d], d, b, packed)
    for m in range(M):
        assert np.array_equal(words(packed)[m, :nw], oracle.pack(k[m], b))
    out = torch.zeros((M, 1008), dtype=torch.int8, device="cuda")[:, :d]
    dq.dq_unpack(packed, d, b, out)
    assert np.array_equal(host(out), k)


@pytest.mark.parametrize("b", [2, 4, 8])
@pytest.mark.parametrize("M,d", [(1, 17), (4, 1000), (16, 20958), (32, 4096), (21, 777), (45, 100003)])
def test_unpack_dequant_sum_bit_exact(dq, b, M, d):
    rng = np.random.default_rng(M * d + b)
    k = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d)).astype(np.int8)
    delta = (rng.random(M) * 1e-2).astype(np.float32)
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    pw = np.zeros((M, ldw), dtype=np.uint32)
    for m in range(M):
        pw[m, :nw] = oracle.pack(k[m], b)
    out = torch.zeros(d, device="cuda")
    scale = float(np.float32(1.0 / M))
    dq.dq_unpack_dequant_sum(dev(pw.view(np.int32)), dev(delta), d, b, scale, out)
    # oracle: the master update with x = 0, g = 0, eta = -1 returns scale * sum_m delta_m k_m
    x = np.zeros(d, dtype=np.float32)
    oracle.master_update(k, delta, np.float32(1.0 / M), np.zeros(d, dtype=np.float32), x, eta=-1.0, l1=0.0)
    assert np.array_equal(host(out), x)


@pytest.mark.parametrize("b", [2, 4, 8])
def test_unpack_dequant_sum_with_extreme_scales(dq, b):
    """Scales that are zero, huge, or so small that a sixteenth of them is not a normal number (the 4-bit decode
    multiplies by delta/16 only where that is exact) still give the oracle's sum bit for bit."""
    M, d = 11, 4099
    rng = np.random.default_rng(b)
    k = rng.integers(-(2 ** (b - 1)), 2 ** (b - 1), size=(M, d)).astype(np.int8)
    delta = np.array([0.0, 2.0 ** -101, 2.0 ** -99, 2.0 ** -120, 2.0 ** -126, 2.0 ** -130, 3e-42, 1.0, 2.0 ** 100, 1e-3,
                      2.0 ** -100], dtype=np.float32)
    nw = dq.packed_words(d, b)
    ldw = (nw + 3) // 4 * 4
    pw = np.zeros((M, ldw), dtype=np.uint32)
    for m in range(M):
        pw[m, :nw] = oracle.pack(k[m], b)
    for order in (np.arange(M), np.arange(M)[::-1].copy()):                 # small terms first, and last
        out = torch.zeros(d, device="cuda")
        dq.dq_unpack_dequant_sum(dev(pw[order].view(np.int32)), dev(delta[order]), d, b, 1.0, out)
        x = np.zeros(d, dtype=np.float32)
        oracle.master_update(k[order], delta[order], np.float32(1.0), np.zeros(d, dtype=np.float32), x, eta=-1.0, l1=0.0)
        assert np.array_equal(host(out).view(np.uint32), x.view(np.uint32))


def test_degenerate_vectors(dq):
    d = 100
    for fill, want_status in [(0.0, 0), (np.nan, 1), (np.inf, 1), (1e-44, 0)]:
        v = np.full(d, fill, dtype=np.float32)
        v[::2] = 0
        packed = torch.full((dq.packed_words(d, 4),), -1, dtype=torch.int32, device="cuda")
        absmax = torch.zeros(1, device="cuda")
        delta = torch.full((1,), 7.0, device="cuda")
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        dq.dq_quantize_pack(dev(v), 4, absmax, False, 1, 1, dq.TAG_GRAD, 0, packed, delta, status)
        k, dlt, st = oracle.quantize(v, 4, 1, 1, 0)
        assert st == want_status == host(status)[0]
        assert not words(packed).any() and not k.any()
        got = host(delta)[0]
        assert (np.isnan(got) and np.isnan(dlt)) or got == dlt


def test_invalid_arguments(dq):
    v = torch.zeros(64, device="cuda")
    a = torch.zeros(1, device="cuda")
    p = torch.zeros(16, dtype=torch.int32, device="cuda")
    for b in (1, 17, 0):
        with pytest.raises(dq.DqError) as e:
            dq.dq_quantize_pack(v, b, a, False, 0, 0, 0, 0, p, a)
        assert e.value.code == dq.ERR_INVALID_ARG
    with pytest.raises(dq.DqError) as e:          # misaligned input
        dq.dq_quantize_pack(v[1:], 4, a, False, 0, 0, 0, 0, p, a)
    assert e.value.code == dq.ERR_INVALID_ARG


def test_determinism_and_stream_independence(dq):
    d, b = 50000, 4
    v = dev(_vec(d, 9))
    outs = []
    for args in [(1, 0, 0), (1, 0, 0), (2, 0, 0), (1, 1, 0), (1, 0, 1)]:
        packed = torch.zeros(dq.packed_words(d, b), dtype=torch.int32, device="cuda")
        dq.dq_quantize_pack(v, b, torch.zeros(1, device="cuda"), False, args[0], args[1], dq.TAG_GRAD, args[2],
                            packed, torch.zeros(1, device="cuda"))
        outs.append(words(packed).copy())
    assert np.array_equal(outs[0], outs[1])
    for o in outs[2:]:
        assert not np.array_equal(outs[0], o)


def test_full_size_vector_sampled(dq):
    """2^28 coordinates in the benchmark's launch shape; the oracle checks sampled windows."""
    N = 1 << 28
    g = torch.Generator(device="cuda").manual_seed(0)
    v = torch.randn(N, device="cuda", generator=g)
    wide = torch.rand(N, device="cuda", generator=g) < 0.1
    v = torch.where(wide, v, v * 0.01).contiguous()
    del wide
    amax_ref = float(v.abs().max().item())
    for b in (8, 4, 2):
        nw = dq.packed_words(N, b)
        packed = torch.zeros(nw, dtype=torch.int32, device="cuda")
        absmax = torch.zeros(1, device="cuda")
        delta = torch.zeros(1, device="cuda")
        dq.dq_quantize_pack(v, b, absmax, False, 42, 3, dq.TAG_GRAD, 11, packed, delta)
        assert host(absmax)[0] == np.float32(amax_ref)
        assert host(delta)[0] == oracle.delta_of(np.float32(amax_ref), b)
        rng = np.random.default_rng(b)
        starts = [0, N - 4096] + [int(s) // 16 * 16 for s in rng.integers(0, N - 4096, size=6)]
        for s in starts:
            seg = host(v[s:s + 4096])
            got = oracle.unpack(words(packed[s * b // 32:(s + 4096) * b // 32]), 4096, b)
            # the oracle quantizes the window plus one coordinate carrying the global max,
            # with the uniforms of the window's true coordinates
            win = np.concatenate([seg, np.array([amax_ref], dtype=np.float32)])
            u = np.concatenate([oracle.uniform_range(42, 3, 11, oracle.TAG_GRAD, s, 4096),
                                np.array([0.5], dtype=np.float32)])
            want, dlt, _ = oracle.quantize_given_uniforms(win, b, u)
            assert dlt == host(delta)[0]
            assert np.array_equal(got, want[:4096])
        del packed


def test_full_size_decode_and_sum_sampled(dq):
    """Alg. 1, master (ii) at the size and in the launch shape of the quantizer benchmark: M = 16 messages of 2^28
    coordinates each (row offsets beyond 4 GB), b in {8, 4, 2}; the messages are the library's own quantization of one
    vector under 16 worker ids, the scales are made distinct.  The oracle unpacks sampled windows of every message,
    aggregates them and must agree bit for bit; the words of two messages are checked against the oracle as well."""
    N, M = 1 << 28, 16
    g = torch.Generator(device="cuda").manual_seed(1)
    v = torch.randn(N, device="cuda", generator=g)
    wide = torch.rand(N, device="cuda", generator=g) < 0.1
    v = torch.where(wide, v, v * 0.01).contiguous()
    del wide
    amax_ref = np.float32(v.abs().max().item())
    absmax = torch.full((1,), float(amax_ref), device="cuda")
    scale = float(np.float32(1.0 / M))
    for b in (8, 4, 2):
        nw = dq.packed_words(N, b)
        packed = torch.zeros((M, nw), dtype=torch.int32, device="cuda")
        delta = torch.zeros(M, device="cuda")
        for w in range(M):
            dq.dq_quantize_pack(v, b, absmax, True, 7, 2, dq.TAG_GRAD, w, packed[w], delta[w:w + 1])
        assert np.all(host(delta) == oracle.delta_of(amax_ref, b))
        delta *= torch.linspace(0.5, 1.5, M, device="cuda")           # distinct scales per message
        res = torch.zeros(N, device="cuda")
        dq.dq_unpack_dequant_sum(packed, delta, N, b, scale, res)
        dl = host(delta)
        rng = np.random.default_rng(100 + b)
        starts = [0, N - 4096] + [int(s) // 16 * 16 for s in rng.integers(0, N - 4096, size=6)]
        for s in starts:
            lo, hi = s * b // 32, (s + 4096) * b // 32
            codes = np.stack([oracle.unpack(words(packed[w, lo:hi]), 4096, b) for w in range(M)])
            x = np.zeros(4096, dtype=np.float32)
            oracle.master_update(codes, dl, np.float32(1.0 / M), np.zeros(4096, dtype=np.float32), x, eta=-1.0, l1=0.0)
            assert np.array_equal(host(res[s:s + 4096]).view(np.uint32), x.view(np.uint32)), (b, s)
            for w in (0, M - 1):                                      # the message itself, against the oracle's quantizer
                win = np.concatenate([host(v[s:s + 4096]), np.array([amax_ref], dtype=np.float32)])
                u = np.concatenate([oracle.uniform_range(7, 2, w, oracle.TAG_GRAD, s, 4096), np.array([0.5], dtype=np.float32)])
                want, _, _ = oracle.quantize_given_uniforms(win, b, u)
                assert np.array_equal(codes[w], want[:4096]), (b, s, w)
        del packed, res
