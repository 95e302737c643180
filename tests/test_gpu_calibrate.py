"""GPU parity of the on-device calibration (MSE grid search for the static per-tensor step, Sec. 3
"Initialization of Quantization Parameters") against the oracle.

The candidate errors are fp32 sums on the GPU and fp64 sums in the oracle: they agree to 1e-4
relative.  The arg-min is compared as a decision: the GPU's candidate must be one whose oracle error
is within 2e-4 of the oracle's minimum (near-ties may legitimately resolve either way); the steps
are bit-exact for unrotated input and within 4 fp32 ulps with rotation.
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


def f32_ulps(a, b):
    ia = np.asarray(a, dtype=np.float32).view(np.int32).astype(np.int64)
    ib = np.asarray(b, dtype=np.float32).view(np.int32).astype(np.int64)
    return np.abs(ia - ib)


@pytest.mark.parametrize("T,K,h,bits,n_grid,gmin", [(16, 512, 1, 4, 10, 0.5), (64, 4096, 1, 4, 50, 0.5),
                                                   (33, 14336, 128, 4, 20, 0.4), (8, 4096, 4096, 4, 16, 0.5),
                                                   (5, 8192, 8192, 8, 12, 0.6), (256, 4096, 1, 8, 24, 0.5),
                                                   (3, 28672, 128, 4, 128, 0.25), (7, 96, 32, 4, 2, 0.5)])
def test_calibration_matches_oracle(pq, T, K, h, bits, n_grid, gmin):
    x = synth.calibration(K, seed=3)[:T] if T <= 256 else synth.activations(T, K, seed=3)
    if T > 2:
        x = x.copy()
        x[0, 0] = np.float16(np.abs(x).max() * 3)          # an outlier, so that clipping can pay
    ref = O.calibrate_mse(x, h, bits, n_grid, gmin)
    res = host(pq.pq_calibrate_static(dev(x), h, bits, n_grid, gmin))
    errs = res[3:].astype(np.float64)
    np.testing.assert_allclose(errs, ref["errs"], rtol=1e-4, atol=1e-12)
    if h <= 1:
        assert res[1] == ref["s_max"]
    else:
        assert f32_ulps(res[1], ref["s_max"]) <= 4
    g = 1.0 - np.arange(n_grid) * (1.0 - np.float64(np.float32(gmin))) / (n_grid - 1)
    best = int(np.argmin(np.abs(g - res[2])))
    assert abs(g[best] - res[2]) < 1e-6
    assert ref["errs"][best] <= ref["errs"].min() * (1 + 2e-4)
    assert f32_ulps(res[0], ref["steps"][best]) <= (0 if h <= 1 else 4)
    assert best == int(np.argmin(errs))                     # the record is consistent with itself


def test_calibration_zero_tensor_and_determinism(pq):
    z = dev(np.zeros((4, 256), dtype=np.float16))
    r = host(pq.pq_calibrate_static(z, 1, 4, 8, 0.5))
    assert r[0] == 1.0 and r[1] == 1.0 and not r[3:].any()
    x = dev(synth.activations(128, 4096, seed=1))
    a = host(pq.pq_calibrate_static(x, 1, 4, 50, 0.5))
    b = host(pq.pq_calibrate_static(x, 1, 4, 50, 0.5))
    assert np.array_equal(a, b)


def test_calibrated_step_feeds_the_layer(pq):
    # the searched step lowers the layer's output error against the unquantized-activation layer
    M, K, N, h = 64, 4096, 512, 1
    x = synth.activations(M, K, seed=11)
    xc = synth.calibration(K, seed=11)
    wq, sw = O.weight_rtn(synth.weights(N, K, seed=11))
    res = host(pq.pq_calibrate_static(dev(xc), h, 4, 50, 0.3))
    exact = x.astype(np.float64) @ (wq.astype(np.float64) * sw.astype(np.float64)[:, None]).T
    err = {}
    for name, s in (("mse", res[0]), ("absmax", res[1])):
        out, _ = pq.pq_linear(dev(x), dev(O.pack(wq)), dev(sw), float(s), h)
        err[name] = np.linalg.norm(host(out).astype(np.float64) - exact)
    assert err["mse"] < err["absmax"]


def test_calibration_argument_errors(pq):
    x = dev(np.ones((2, 256), dtype=np.float16))
    for kw, status in ((dict(n_grid=1), 2), (dict(n_grid=129), 2), (dict(bits=5), 2), (dict(gamma_min=1.0), 4),
                       (dict(gamma_min=0.0), 4)):
        args = dict(had_block=1, bits=4, n_grid=8, gamma_min=0.5)
        args.update(kw)
        with pytest.raises(pq.PQError) as e:
            pq.pq_calibrate_static(x, args["had_block"], args["bits"], args["n_grid"], args["gamma_min"])
        assert e.value.status == status, kw
