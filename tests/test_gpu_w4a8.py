"""GPU parity of the W4A8 calls (8-bit static activations, Table 3's W4A8 rows) against the oracle.

Same two gates as the 4-bit path: codes bit-exact for unrotated input, accumulators bit-exact,
output within one fp16 ulp of the oracle's epilogue; end to end, codes may differ only at
rounding ties (at most 0.1 % of them, |t - (k + 1/2)| <= 1e-3) and the output's max error is at
most 1e-2 of max|out|.
"""

import numpy as np
import pytest
import torch

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import dev, host, ulp_diff

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


def codes_of(t):
    return O.ungroup_even_odd(host(t))


# ------------------------------------------------------------------ codes
@pytest.mark.parametrize("scale", [0.25, 0.1, 1.0 / 3.0, 0.0123, 1.7, 3e-5, 41.0, 517.0])
def test_codes8_exact_for_every_fp16_value(pq, scale):
    v = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    x = v[np.isfinite(v)].reshape(31, 2048)
    s = np.float32(scale)
    got = codes_of(pq.pq_rotate_quant8(dev(x), 1, float(s)))
    assert np.array_equal(got, O.quantize_bits(x, s, 8))


def test_codes8_exact_at_ties(pq):
    rng = np.random.default_rng(17)
    for trial in range(6):
        s = np.float32(rng.uniform(0.001, 0.5))
        k = rng.integers(-130, 130, size=(8, 1024)).astype(np.float64)
        x = ((k + 0.5) * np.float64(s)).astype(np.float16)
        got = codes_of(pq.pq_rotate_quant8(dev(x), 0, float(s)))
        assert np.array_equal(got, O.quantize_bits(x, s, 8)), "step %r" % s


@pytest.mark.parametrize("M,K,h", [(5, 128, 1), (16, 512, 512), (33, 4096, 128), (3, 14336, 128), (5, 4096, 4096),
                                   (2, 8192, 8192), (3, 16384, 16384), (258, 1024, 64)])
def test_codes8_rotated(pq, M, K, h):
    x = synth.activations(M, K, seed=2)
    sx = O.calibrate_absmax(synth.calibration(K, seed=2), h, 8)
    y = O.rotate(x, h)
    want = O.quantize_bits(y, sx, 8)
    got = codes_of(pq.pq_rotate_quant8(dev(x), h, float(sx)))
    diff = got.astype(np.int32) - want.astype(np.int32)
    idx = np.nonzero(diff)
    if h <= 1:
        assert idx[0].size == 0
        return
    assert idx[0].size <= 1e-3 * diff.size
    if idx[0].size:
        assert np.all(np.abs(diff[idx]) == 1)
        t = y[idx] / np.float64(sx)
        lo = np.minimum(got[idx], want[idx]).astype(np.float64)
        assert np.all(np.abs(t - (lo + 0.5)) <= 1e-3)


# ------------------------------------------------------------------ product + epilogue
SHAPES = [(16, 512, 512), (1, 128, 128), (3, 48, 256), (5, 272, 384), (64, 128, 128), (255, 400, 1152),
          (257, 512, 2048), (130, 1040, 14336), (2047, 256, 512), (300, 6144, 512), (513, 768, 1024),
          (1900, 14336, 128), (2048, 14336, 256)]      # the last two: one launch mixes 256- and 192-wide tiles


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_w4a8_product_and_epilogue(pq, M, N, K):
    q = synth.random_codes(M, K, seed=M + K, stream=8, lo=-128, hi=127)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.01373)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    out_ref = O.epilogue(acc_ref, sx, sw)
    out, acc = pq.pq_w4a8_gemm(dev(O.group_even_odd(q)), dev(wq), dev(sw), float(sx), want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), out_ref).max() <= 1
    out2, _ = pq.pq_w4a8_gemm(dev(O.group_even_odd(q)), dev(wq), dev(sw), float(sx))
    assert np.array_equal(host(out2), host(out))


@pytest.mark.parametrize("M", [1, 2, 4, 5, 8])
@pytest.mark.parametrize("N,K", [(512, 512), (1024, 14336), (4608, 16384), (6144, 4096), (256, 28672), (48, 2176)])
def test_w4a8_decode_sizes(pq, M, N, K):
    """M <= 8 streams the weights once (4-way byte dot products); long rows that do not fit LDS fall back."""
    q = synth.random_codes(M, K, seed=M + K, stream=8, lo=-128, hi=127)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.0213)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    out, acc = pq.pq_w4a8_gemm(dev(O.group_even_odd(q)), dev(wq), dev(sw), float(sx), want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, sx, sw)).max() <= 1
    prev = pq.pq_set_gemm_variant(2)                       # the tiled kernel gives the same accumulators
    try:
        _, acc2 = pq.pq_w4a8_gemm(dev(O.group_even_odd(q)), dev(wq), dev(sw), float(sx), want_out=False, want_acc=True)
    finally:
        pq.pq_set_gemm_variant(prev)
    assert np.array_equal(host(acc2), host(acc))


@pytest.mark.parametrize("a,w", [(-128, -8), (-128, 7), (127, -8), (127, 7)])
def test_w4a8_extreme_codes_longest_row(pq, a, w):
    M, N, K = 4, 32, 65536
    q = np.full((M, K), a, dtype=np.int8)
    wc = np.full((N, K), w, dtype=np.int8)
    sw = np.full(N, 2.0 ** -20, dtype=np.float32)
    out, acc = pq.pq_w4a8_gemm(dev(q), dev(O.pack(wc)), dev(sw), 1.0, want_out=True, want_acc=True)
    assert np.all(host(acc) == a * w * K)
    assert ulp_diff(host(out), O.epilogue(np.full((M, N), a * w * K, dtype=np.int64), np.float32(1), sw)).max() <= 1


# ------------------------------------------------------------------ end to end
@pytest.mark.parametrize("M,K,N,h", [(48, 512, 512, 1), (33, 1024, 768, 128), (300, 4096, 1024, 1),
                                     (70, 14336, 512, 128), (4, 4096, 4096, 1), (1, 2048, 256, 2048)])
def test_linear_w4a8(pq, M, K, N, h):
    x = synth.activations(M, K, seed=3)
    wq, sw = O.weight_rtn(synth.weights(N, K, seed=3))
    sx = O.calibrate_absmax(synth.calibration(K, seed=3), h, 8)
    wp = O.pack(wq)
    ref = O.linear_bits(x, wp, sw, sx, h, 8)
    out, ws = pq.pq_linear_w4a8(dev(x), dev(wp), dev(sw), float(sx), h)
    got_q = O.ungroup_even_odd(host(ws)[: M * K].view(np.int8).reshape(M, K))
    diff = got_q.astype(np.int32) - ref["q"].astype(np.int32)
    idx = np.nonzero(diff)
    assert idx[0].size <= 1e-3 * diff.size
    if idx[0].size:
        assert h > 1 and np.all(np.abs(diff[idx]) == 1)
        t = ref["y"][idx] / np.float64(sx)
        lo = np.minimum(got_q[idx], ref["q"][idx]).astype(np.float64)
        assert np.all(np.abs(t - (lo + 0.5)) <= 1e-3)
    o_ref = ref["out"].astype(np.float64)
    rel = np.max(np.abs(host(out).astype(np.float64) - o_ref)) / np.max(np.abs(o_ref))
    assert rel <= 1e-2
    sub = O.epilogue(O.gemm_i64(got_q, wq), np.float32(sx), sw)
    assert ulp_diff(sub, host(out)).max() <= 1


def test_w4a8_argument_errors(pq):
    x = dev(np.zeros((4, 160), dtype=np.float16))
    with pytest.raises(pq.PQError) as e:
        pq.pq_rotate_quant8(x, 1, 1.0)                      # K % 128 != 0
    assert e.value.status == 2
    q = dev(np.zeros((4, 160), dtype=np.int8))
    w = dev(np.zeros((16, 80), dtype=np.uint8))
    sw = dev(np.ones(16, dtype=np.float32))
    with pytest.raises(pq.PQError) as e:
        pq.pq_w4a8_gemm(q, w, sw, 1.0)
    assert e.value.status == 2
    buf = torch.full((2, 128), 5, dtype=torch.int8, device="cuda")
    x2 = dev(np.ones((2, 128), dtype=np.float16))
    import ctypes
    rc = pq.lib().pq_rotate_quant8(ctypes.c_void_p(x2.data_ptr()), 0, 128, 1, 1.0, ctypes.c_void_p(buf.data_ptr()),
                                   None)                                                  # M = 0: no-op
    assert rc == 0
    torch.cuda.synchronize()
    assert bool((buf == 5).all())
