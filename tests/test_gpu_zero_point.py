"""GPU parity of the static quantizer with a zero-point (Eq. 1 in its general form) against the oracle:
codes bit-exact for unrotated input (ties included) and differing only at ties with rotation; the
correction vector and the raw accumulators bit-exact; outputs within one fp16 ulp of the oracle's
epilogue on (acc + correction); end to end within 1e-2 of max|out|."""

import numpy as np
import pytest

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import dev, host, ulp_diff

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


def stored(u):
    return (u.astype(np.int16) - 8).astype(np.int8)


@pytest.mark.parametrize("z", [0, 3, 8, 11, 15])
@pytest.mark.parametrize("scale", [0.25, 0.1, 1.0 / 3.0, 0.0123, 41.0])
def test_zp_codes_exact_for_every_fp16_value(pq, z, scale):
    v = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    x = v[np.isfinite(v)].reshape(31, 2048)
    s = np.float32(scale)
    got = O.unpack(host(pq.pq_rotate_quant_zp(dev(x), 1, float(s), z)))
    assert np.array_equal(got, stored(O.quantize_zp(x, s, z)))


def test_zp_codes_exact_at_ties(pq):
    rng = np.random.default_rng(19)
    for z in (1, 6, 13):
        s = np.float32(rng.uniform(0.01, 2.0))
        k = rng.integers(-17, 17, size=(8, 1024)).astype(np.float64)
        x = ((k + 0.5) * np.float64(s)).astype(np.float16)
        got = O.unpack(host(pq.pq_rotate_quant_zp(dev(x), 0, float(s), z)))
        assert np.array_equal(got, stored(O.quantize_zp(x, s, z))), (z, s)


@pytest.mark.parametrize("M,K,h", [(16, 512, 512), (33, 14336, 128), (5, 4096, 4096), (2, 8192, 8192), (300, 1024, 64)])
def test_zp_codes_rotated(pq, M, K, h):
    x = np.abs(synth.activations(M, K, seed=51)) if h <= 64 else synth.activations(M, K, seed=51)
    y = O.rotate(x, h)
    s, z = O.minmax_params(O.rotate(synth.calibration(K, seed=51), h))
    want = stored(O.quantize_zp(y, s, z))
    got = O.unpack(host(pq.pq_rotate_quant_zp(dev(x), h, float(s), z)))
    d = np.nonzero(got != want)
    assert d[0].size <= 1e-3 * got.size
    if d[0].size:
        assert np.all(np.abs(got[d].astype(int) - want[d]) == 1)
        t = y[d] / np.float64(s) + z - 8
        assert np.all(np.abs(t - (np.minimum(got[d], want[d]) + 0.5)) <= 1e-3)


@pytest.mark.parametrize("N,K,z", [(512, 512, 0), (272, 384, 5), (4096, 14336, 15), (48, 32, 8), (6144, 4096, 11)])
def test_zero_point_correction_exact(pq, N, K, z):
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    got = host(pq.pq_zero_point_correction(dev(wq), z))
    assert np.array_equal(got.astype(np.int64), (8 - z) * O.unpack(wq).astype(np.int64).sum(axis=1))


@pytest.mark.parametrize("M,N,K,z", [(16, 512, 512, 3), (1, 128, 128, 0), (5, 272, 384, 15), (8, 1024, 14336, 6),
                                     (255, 400, 1152, 11), (257, 512, 2048, 1), (130, 1040, 14336, 13),
                                     (1030, 14336, 128, 5), (2048, 14336, 128, 9), (40, 64, 32768, 0)])
def test_zp_product_and_epilogue(pq, M, N, K, z):
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.173)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    corr = (8 - z) * O.unpack(wq).astype(np.int64).sum(axis=1)
    d_corr = pq.pq_zero_point_correction(dev(wq), z)
    out, acc = pq.pq_w4a4_gemm_zp(dev(xq), dev(wq), dev(sw), float(sx), d_corr, want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref + corr[None, :], sx, sw)).max() <= 1


def test_zp_extreme_codes(pq):
    # every activation at X_INT = 15 with z = 0 and every weight at -8, longest supported row
    M, N, K = 3, 32, 32768
    xq = np.full((M, K // 2), 0x77, np.uint8)
    wq = np.full((N, K // 2), 0x88, np.uint8)
    sw = np.full(N, 2.0 ** -12, np.float32)
    d_corr = pq.pq_zero_point_correction(dev(wq), 0)
    out, acc = pq.pq_w4a4_gemm_zp(dev(xq), dev(wq), dev(sw), 1.0, d_corr, want_out=True, want_acc=True)
    assert np.all(host(acc) == -56 * K) and np.all(host(d_corr) == -64 * K)
    assert ulp_diff(host(out), O.epilogue(np.full((M, N), -120 * K, np.int64), np.float32(1), sw)).max() <= 1


@pytest.mark.parametrize("M,K,N,h", [(48, 512, 512, 1), (300, 4096, 1024, 1), (70, 14336, 512, 128), (4, 4096, 4096, 1)])
def test_zp_layer_end_to_end(pq, M, K, N, h):
    # one-sided activations (as after a gate): this is where a zero-point pays
    x = np.abs(synth.activations(M, K, seed=52)) if h == 1 else synth.activations(M, K, seed=52)
    wq, sw = O.weight_rtn(synth.weights(N, K, seed=52))
    xc = np.abs(synth.calibration(K, seed=52)) if h == 1 else synth.calibration(K, seed=52)
    s, z = O.minmax_params(O.rotate(xc, h))
    ref = O.linear_zp(x, O.pack(wq), sw, s, z, h)
    d_w = dev(O.pack(wq))
    xq = pq.pq_rotate_quant_zp(dev(x), h, float(s), z)
    out, _ = pq.pq_w4a4_gemm_zp(xq, d_w, dev(sw), float(s), pq.pq_zero_point_correction(d_w, z))
    got_c = O.unpack(host(xq))
    d = np.nonzero(got_c != ref["codes"])
    assert d[0].size <= 1e-3 * got_c.size and (h > 1 or d[0].size == 0)
    o_ref = ref["out"].astype(np.float64)
    assert np.abs(host(out).astype(np.float64) - o_ref).max() <= 1e-2 * np.abs(o_ref).max()
    sub = O.epilogue(O.gemm_i64(got_c, wq) + ref["corr"][None, :], s, sw)
    assert ulp_diff(sub, host(out)).max() <= 1
    if h == 1:
        # against the unquantized-activation layer the zero-point beats the symmetric quantizer on one-sided data
        exact = x.astype(np.float64) @ (wq.astype(np.float64) * sw.astype(np.float64)[:, None]).T
        s_sym = np.float32(np.abs(xc.astype(np.float64)).max() / 7)
        o_sym, _ = pq.pq_linear(dev(x), d_w, dev(sw), float(s_sym), 1)
        assert np.linalg.norm(host(out) - exact) < 0.7 * np.linalg.norm(host(o_sym) - exact)


def test_zp_argument_errors(pq):
    x = dev(np.ones((2, 256), dtype=np.float16))
    for z in (-1, 16):
        with pytest.raises(pq.PQError) as e:
            pq.pq_rotate_quant_zp(x, 1, 1.0, z)
        assert e.value.status == 2
    with pytest.raises(pq.PQError) as e:
        pq.pq_zero_point_correction(dev(np.zeros((16, 128), np.uint8)), 16)
    assert e.value.status == 2
