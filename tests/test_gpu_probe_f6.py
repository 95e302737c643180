"""The 6-bit floating-point matrix instruction as an exact integer multiplier (pq_probe_f6_product):
4-bit codes written as E3M2 floats, fp32 accumulation, against the oracle's int64 sums.  This is a
property of the GPU that a later kernel can build on; the probe is a service call, not the path."""

import numpy as np
import pytest
import torch

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


@pytest.mark.parametrize("K", [64, 128, 4096, 14336, 65536, 262080])
def test_random_codes_are_multiplied_exactly(pq, K):
    a = synth.random_codes(32, K, seed=K, stream=4)
    b = synth.random_codes(32, K, seed=K, stream=8)
    got = host(pq.pq_probe_f6_product(dev(a), dev(b)))
    assert np.array_equal(got.astype(np.int64), O.gemm_i64(a, b))


@pytest.mark.parametrize("va,vb", [(-8, -8), (-8, 7), (7, 7), (8, 8), (8, -8), (1, -1), (0, 5)])
def test_constant_codes_up_to_the_largest_sum(pq, va, vb):
    K = 262080                                   # 64 K = 16 773 120 < 2^24
    a = np.full((32, K), va, np.int8)
    b = np.full((32, K), vb, np.int8)
    got = host(pq.pq_probe_f6_product(dev(a), dev(b)))
    assert (got == va * vb * K).all()


def test_every_pair_of_codes(pq):
    """Row i of a is the code i - 8 (17 values, -8..8) in channel 0 and zero elsewhere, likewise b: the
    32 x 32 outputs hold every product of two codes."""
    a = np.zeros((32, 64), np.int8)
    a[:17, 0] = np.arange(-8, 9)
    got = host(pq.pq_probe_f6_product(dev(a), dev(a)))
    want = np.outer(a[:, 0].astype(np.int64), a[:, 0].astype(np.int64))
    assert np.array_equal(got.astype(np.int64), want)


def test_out_of_range_codes_are_clamped_and_bad_shapes_refused(pq):
    a = np.full((32, 64), 100, np.int8)
    b = np.full((32, 64), -100, np.int8)
    assert (host(pq.pq_probe_f6_product(dev(a), dev(b))) == -64 * 64).all()
    with pytest.raises(pq.PQError, match="PQ_ERR_SHAPE"):
        pq.pq_probe_f6_product(dev(np.zeros((32, 96), np.int8)), dev(np.zeros((32, 96), np.int8)))


def test_rate_probe_runs(pq):
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    ops = pq.pq_probe_mfma_f6(torch.zeros(4096, dtype=torch.uint8, device="cuda"), 10, 8, sink)
    torch.cuda.synchronize()
    assert ops == 8 * 4 * 10 * 16 * 131072 and int(sink[0]) == 0
