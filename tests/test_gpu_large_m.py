"""Many tokens: more rows than one launch's grid takes (the quantizer kernels split at 65534 rows),
and the matrix kernel with hundreds of row tiles.  Small K keeps the oracle fast."""

import numpy as np
import pytest

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import dev, host, ulp_diff

pytestmark = pytest.mark.gpu

M_BIG = 2 * 65534 + 3


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


def test_quantizers_over_the_row_limit(pq):
    K = 128
    x = synth.activations(M_BIG, K, seed=41)
    s = np.float32(0.37)
    assert np.array_equal(host(pq.pq_rotate_quant(dev(x), 1, float(s))), O.pack(O.quantize(x, s)))
    assert np.array_equal(O.ungroup_even_odd(host(pq.pq_rotate_quant8(dev(x), 1, float(s) / 16))),
                          O.quantize_bits(x, s / np.float32(16), 8))
    y = O.rotate(x, 128)
    got = O.unpack(host(pq.pq_rotate_quant(dev(x), 128, float(s))))
    want = O.quantize(y, s)
    d = np.nonzero(got != want)
    assert d[0].size <= 1e-3 * got.size
    assert np.all(np.abs(y[d] / np.float64(s) - (np.minimum(got[d], want[d]) + 0.5)) <= 1e-3)
    yf = host(pq.pq_rotate_f16(dev(x), 128))
    near = np.abs(yf.astype(np.float64) - y) <= 7 * 2.0 ** -23 * np.abs(y).max() + 2.0 ** -11 * np.abs(y)
    assert np.all((ulp_diff(yf, y.astype(np.float16)) <= 1) | near)        # near zero: absolute fp32 butterfly error
    hs = np.array([0.21], dtype=np.float32)
    assert np.array_equal(O.unpack(host(pq.pq_rotate_quant_heads(dev(x), 1, False, dev(hs)))), O.quantize_heads(x, hs, 128))
    q, st = pq.pq_rotate_quant_dynamic(dev(x), 1, 1.0, 4)
    wq, ws = O.quantize_dynamic(x, 1.0, 4)
    assert np.array_equal(host(st), ws) and np.array_equal(O.unpack(host(q)), wq)


def test_gemm_many_row_tiles(pq):
    M, N, K = 70001, 48, 128
    xq = synth.random_packed(M, K, seed=42)
    wq = synth.random_packed(N, K, seed=43, stream=7)
    sw = synth.random_scales(N, seed=44)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.125, want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.125), sw)).max() <= 1


def test_fused_producers_over_the_row_limit(pq):
    K = 128
    g, u = synth.activations(M_BIG, K, seed=45), synth.activations(M_BIG, K, seed=46)
    y = O.rotate(O.silu_mul(g, u), 128)
    s = np.float32(np.abs(y).max() / 7)
    got = O.unpack(host(pq.pq_silu_mul_rotate_quant(dev(g), dev(u), 128, float(s))))
    want = O.quantize(y, s)
    d = np.nonzero(got != want)
    assert d[0].size <= 1e-3 * got.size
    assert np.all(np.abs(y[d] / np.float64(s) - (np.minimum(got[d], want[d]) + 0.5)) <= 1e-3)
    yn = O.rmsnorm(g, 1e-5)
    got = O.unpack(host(pq.pq_rmsnorm_quant(dev(g), 1e-5, 0.4)))
    want = O.quantize(yn, np.float32(0.4))
    d = np.nonzero(got != want)
    assert d[0].size <= 1e-3 * got.size
    assert np.all(np.abs(yn[d] / np.float64(np.float32(0.4)) - (np.minimum(got[d], want[d]) + 0.5)) <= 1e-3)
