"""GPU parity of the fused producers (silu(gate) * up -> rotate -> quantize for down_proj;
RMS normalisation -> quantize for q/k/v/gate/up) against the oracle.

The producers are evaluated in fp32 on the GPU and fp64 in the oracle, so codes may differ only at
rounding ties: at most 0.1 % of them, each by 1, and only where |t - (k + 1/2)| <= 1e-3.
"""

import numpy as np
import pytest

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


def check(got, y, s):
    want = O.quantize(y, s)
    diff = got.astype(np.int32) - want.astype(np.int32)
    idx = np.nonzero(diff)
    assert idx[0].size <= 1e-3 * diff.size
    if idx[0].size:
        assert np.all(np.abs(diff[idx]) == 1)
        t = y[idx] / np.float64(s)
        lo = np.minimum(got[idx], want[idx]).astype(np.float64)
        assert np.all(np.abs(t - (lo + 0.5)) <= 1e-3)
    return idx[0].size


@pytest.mark.parametrize("M,K,h", [(16, 512, 128), (33, 14336, 128), (5, 11008, 128), (300, 1024, 64), (3, 4096, 4096),
                                   (2, 8192, 8192), (3, 16384, 16384), (7, 512, 1), (2049, 256, 128)])
def test_silu_mul_rotate_quant(pq, M, K, h):
    g = synth.activations(M, K, seed=31)
    u = synth.activations(M, K, seed=32)
    gc, uc = synth.calibration(K, seed=31), synth.calibration(K, seed=32)
    sx = np.float32(np.abs(O.rotate(O.silu_mul(gc, uc), h)).max() / 7)
    y = O.rotate(O.silu_mul(g, u), h)
    got = O.unpack(host(pq.pq_silu_mul_rotate_quant(dev(g), dev(u), h, float(sx))))
    check(got, y, sx)
    # the unfused pair (producer rounded to fp16, then pq_rotate_quant) gives nearly the same codes
    x16 = O.silu_mul(g, u).astype(np.float16)
    if h == 1:
        return
    unf = O.unpack(host(pq.pq_rotate_quant(dev(x16), h, float(sx))))
    assert (unf != got).mean() <= 2e-2                      # same tensor up to the fp16 rounding of x


@pytest.mark.parametrize("M,K,eps", [(16, 512, 1e-5), (33, 4096, 1e-5), (5, 14336, 1e-6), (300, 1024, 0.0),
                                     (3, 28672, 1e-5), (2, 32768, 1e-5), (7, 96, 1e-5), (2049, 256, 1e-5)])
def test_rmsnorm_quant(pq, M, K, eps):
    x = synth.activations(M, K, seed=33)
    sx = np.float32(np.abs(O.rmsnorm(synth.calibration(K, seed=33), eps)).max() / 7)
    y = O.rmsnorm(x, np.float32(eps))
    got = O.unpack(host(pq.pq_rmsnorm_quant(dev(x), eps, float(sx))))
    check(got, y, sx)


def test_rmsnorm_quant_zero_row_and_scale_invariance(pq):
    x = synth.activations(8, 1024, seed=34)
    x[3] = 0
    a = O.unpack(host(pq.pq_rmsnorm_quant(dev(x), 1e-5, 0.4)))
    assert not a[3].any()
    b = O.unpack(host(pq.pq_rmsnorm_quant(dev((x * np.float16(4.0)).astype(np.float16)), 1e-5 * 16, 0.4)))
    assert np.array_equal(a, b)                             # powers of two scale exactly: identical codes


def test_fusion_feeds_the_layer(pq):
    # silu-gated down_proj end to end: fused quantizer + GEMM against the oracle on the same codes
    M, K, N, h = 40, 14336, 256, 128
    g, u = synth.activations(M, K, seed=35), synth.activations(M, K, seed=36)
    wq, sw = O.weight_rtn(synth.weights(N, K, seed=35))
    y = O.rotate(O.silu_mul(g, u), h)
    sx = np.float32(np.abs(y).max() / 7)
    xq = pq.pq_silu_mul_rotate_quant(dev(g), dev(u), h, float(sx))
    out, _ = pq.pq_w4a4_gemm(xq, dev(O.pack(wq)), dev(sw), float(sx))
    ref = O.epilogue(O.gemm_i64(O.quantize(y, sx), wq), sx, sw).astype(np.float64)
    rel = np.abs(host(out).astype(np.float64) - ref).max() / np.abs(ref).max()
    assert rel <= 1e-2


def test_fusion_argument_errors(pq):
    g = dev(np.ones((2, 256), dtype=np.float16))
    with pytest.raises(pq.PQError) as e:
        pq.pq_silu_mul_rotate_quant(g, g, 96, 1.0)
    assert e.value.status == 2
    with pytest.raises(pq.PQError) as e:
        pq.pq_rmsnorm_quant(g, -1.0, 1.0)
    assert e.value.status == 4
    with pytest.raises(pq.PQError) as e:
        pq.pq_rmsnorm_quant(g, 1e-5, 0.0)
    assert e.value.status == 4
