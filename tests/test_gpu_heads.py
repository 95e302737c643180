"""GPU parity of the attention-side calls: online R3 (head-wise rotation of queries and keys) and
per-head static KV-cache quantization (App. B "Online Rotation"; Table 1 row O2).

Unrotated input (values): codes bit-exact.  Rotated input (keys): codes may differ from the fp64
oracle only at rounding ties (at most 0.1 %, |t - (k + 1/2)| <= 1e-3).  Rotation to fp16 (queries):
fp32 butterflies and one rounding, so at most one fp16 ulp from the oracle's rounded fp64 result
(or, for outputs near zero, within the absolute error of the fp32 butterflies), and equal for at
least 99.8 % of the elements.
"""

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


def head_steps(K, H, D, rotate, seed):
    """Static per-head steps from a separate calibration batch: max|y_head| / 7."""
    yc = O.rotate(synth.calibration(K, seed), D if rotate else 1)
    return (np.abs(yc).reshape(-1, H, D).max(axis=(0, 2)) / 7.0).astype(np.float32)


@pytest.mark.parametrize("T,H,D", [(33, 8, 128), (7, 32, 128), (300, 8, 64), (5, 4, 256), (2, 96, 32), (3, 3, 2048),
                                   (2049, 8, 128)])
def test_values_per_head_codes_exact(pq, T, H, D):
    K = H * D
    x = synth.activations(T, K, seed=7)
    s = head_steps(K, H, D, False, 7)
    got = O.unpack(host(pq.pq_rotate_quant_heads(dev(x), H, False, dev(s))))
    assert np.array_equal(got, O.quantize_heads(x, s, D))


@pytest.mark.parametrize("T,H,D", [(33, 8, 128), (7, 32, 128), (300, 8, 64), (5, 4, 256), (2, 96, 32), (3, 3, 2048),
                                   (3, 2, 1024)])
def test_keys_rotated_per_head_codes(pq, T, H, D):
    K = H * D
    x = synth.activations(T, K, seed=8)
    s = head_steps(K, H, D, True, 8)
    y = O.rotate(x, D)
    want = O.quantize_heads(y, s, D)
    got = O.unpack(host(pq.pq_rotate_quant_heads(dev(x), H, True, dev(s))))
    diff = got.astype(np.int32) - want.astype(np.int32)
    idx = np.nonzero(diff)
    assert idx[0].size <= 1e-3 * diff.size
    if idx[0].size:
        assert np.all(np.abs(diff[idx]) == 1)
        t = y[idx] / np.repeat(s.astype(np.float64), D)[idx[1]]
        lo = np.minimum(got[idx], want[idx]).astype(np.float64)
        assert np.all(np.abs(t - (lo + 0.5)) <= 1e-3)


def test_per_head_ties_exact(pq):
    # values exactly on (k + 1/2) * s for head steps that are not powers of two
    rng = np.random.default_rng(3)
    H, D, T = 8, 128, 16
    s = rng.uniform(0.01, 2.0, size=H).astype(np.float32)
    k = rng.integers(-9, 9, size=(T, H * D)).astype(np.float64)
    x = ((k + 0.5) * np.repeat(s.astype(np.float64), D)[None, :]).astype(np.float16)
    got = O.unpack(host(pq.pq_rotate_quant_heads(dev(x), H, False, dev(s))))
    assert np.array_equal(got, O.quantize_heads(x, s, D))


@pytest.mark.parametrize("M,K,h", [(33, 4096, 128), (300, 1024, 64), (5, 4096, 4096), (3, 16384, 16384), (2, 8192, 2048),
                                   (9, 96, 32), (2049, 1024, 128)])
def test_rotate_to_fp16(pq, M, K, h):
    x = synth.activations(M, K, seed=9)
    want = O.rotate(x, h).astype(np.float16)
    got = host(pq.pq_rotate_f16(dev(x), h))
    d = ulp_diff(got, want)
    # log2(h) fp32 butterfly stages, each within 2^-24 relative of values no larger than sqrt(h) max|y|:
    # an absolute error that exceeds one fp16 ulp only for outputs near zero
    tol = np.log2(h) * 2.0 ** -23 * np.abs(want.astype(np.float64)).max()
    near = np.abs(got.astype(np.float64) - want.astype(np.float64)) <= tol
    assert np.all((d <= 1) | near)
    assert (d != 0).mean() <= 2e-3
    # the rotation is an involution: applying it twice returns x up to two fp16 roundings
    back = host(pq.pq_rotate_f16(dev(got), h)).astype(np.float64)
    err = np.abs(back - x.astype(np.float64)).max()
    assert err <= 2.0 ** -9 * np.abs(x.astype(np.float64)).max()


def test_heads_argument_errors(pq):
    x = dev(np.ones((2, 96), dtype=np.float16))
    s = dev(np.ones(3, dtype=np.float32))
    with pytest.raises(pq.PQError) as e:
        pq.pq_rotate_quant_heads(dev(np.ones((2, 48), dtype=np.float16)), 3, True, s)    # head_dim 16 < 32
    assert e.value.status == 2
    with pytest.raises(pq.PQError) as e:
        pq.pq_rotate_quant_heads(dev(np.ones((2, 288), dtype=np.float16)), 3, True, s)   # head_dim 96: not 2^n
    assert e.value.status == 2
    with pytest.raises(pq.PQError) as e:
        pq.pq_rotate_f16(x, 1)
    assert e.value.status == 2
    with pytest.raises(pq.PQError) as e:
        pq.pq_rotate_f16(x, 64)                                                           # 96 % 64 != 0
    assert e.value.status == 2
    out = pq.pq_rotate_quant_heads(x, 3, False, s)
    assert np.array_equal(O.unpack(host(out)), np.ones((2, 96), dtype=np.int8))


def f32_ulps(a, b):
    ia = np.asarray(a, dtype=np.float32).view(np.int32).astype(np.int64)
    ib = np.asarray(b, dtype=np.float32).view(np.int32).astype(np.int64)
    return np.abs(ia - ib)


@pytest.mark.parametrize("group", [32, 64, 128])
@pytest.mark.parametrize("T,H,D,clip", [(33, 8, 128, 1.0), (7, 32, 128, 0.875), (300, 2, 256, 1.0), (2049, 8, 128, 1.0)])
def test_groups_dynamic_values_exact(pq, group, T, H, D, clip):
    x = synth.activations(T, H * D, seed=61)
    if T > 2:
        x[1, :group] = 0
    want_q, want_s = O.quantize_groups_dynamic(x, group, clip)
    q, s = pq.pq_rotate_quant_groups(dev(x), H, False, group, clip)
    assert np.array_equal(host(s), want_s)
    assert np.array_equal(O.unpack(host(q)), want_q)


@pytest.mark.parametrize("group", [32, 128])
@pytest.mark.parametrize("T,H,D", [(33, 8, 128), (7, 32, 128), (5, 4, 256), (3, 3, 2048)])
def test_groups_dynamic_keys_rotated(pq, group, T, H, D):
    x = synth.activations(T, H * D, seed=62)
    y = O.rotate(x, D)
    want_q, want_s = O.quantize_groups_dynamic(y, group)
    q, s = pq.pq_rotate_quant_groups(dev(x), H, True, group, 1.0)
    assert f32_ulps(host(s), want_s).max() <= 4
    got = O.unpack(host(q))
    d = np.nonzero(got != want_q)
    assert d[0].size <= 1e-3 * got.size
    if d[0].size:
        t = y[d] / want_s.astype(np.float64)[d[0], d[1] // group]
        assert np.all(np.abs(got[d].astype(int) - want_q[d]) == 1)
        assert np.all(np.abs(t - (np.minimum(got[d], want_q[d]) + 0.5)) <= 1e-3)


def test_groups_argument_errors(pq):
    x = dev(np.ones((2, 256), dtype=np.float16))
    with pytest.raises(pq.PQError) as e:
        pq.pq_rotate_quant_groups(x, 2, True, 48)
    assert e.value.status == 2
    with pytest.raises(pq.PQError) as e:
        pq.pq_rotate_quant_groups(dev(np.ones((2, 128), dtype=np.float16)), 2, True, 128)      # head_dim 64 < group
    assert e.value.status == 2
    with pytest.raises(pq.PQError) as e:
        pq.pq_rotate_quant_groups(x, 2, True, 64, 0.0)
    assert e.value.status == 4
