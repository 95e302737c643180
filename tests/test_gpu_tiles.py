"""Every tile configuration of the tiled product, forced one by one (pq_set_gemm_tile):
the automatic choice picks a configuration from the shape, so a given test shape exercises one of
them; here each is run on shapes with ragged last tiles in both directions, one and several
128-channel stages, and the mixed-width launch, against the oracle's integer sums and its epilogue.
"""

import os

import numpy as np
import pytest

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import dev, host, ulp_diff

pytestmark = pytest.mark.gpu

TILES = {0: "256x256", 1: "256x128", 2: "128x128", 3: "256x192", 4: "64x128", 5: "256x256, 8 wavefronts",
         6: "256x256, 4-stage ring", 7: "256x128, 4x2 wavefronts", 8: "256x128, 2x4 wavefronts"}


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


@pytest.fixture
def tile_env(pq):
    saved = pq.pq_set_gemm_tile(-1)
    yield
    pq.pq_set_gemm_tile(saved)


@pytest.mark.parametrize("tile", sorted(TILES))
@pytest.mark.parametrize("M,N,K", [(300, 400, 1152), (64, 128, 128), (517, 784, 384), (129, 1040, 2048)])
def test_forced_tile_configuration(pq, tile_env, tile, M, N, K):
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.0917)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    pq.pq_set_gemm_tile(tile)
    prev = pq.pq_set_gemm_variant(2)
    try:
        out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), float(sx), want_out=True, want_acc=True)
    finally:
        pq.pq_set_gemm_variant(prev)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref), TILES[tile]
    assert ulp_diff(host(out), O.epilogue(acc_ref, sx, sw)).max() <= 1, TILES[tile]


@pytest.mark.parametrize("tile", [1, 2, 3, 4])
def test_forced_tile_int8_activations_and_per_token_steps(pq, tile_env, tile):
    M, N, K = 300, 400, 1152
    q = synth.random_codes(M, K, seed=5, stream=9, lo=-128, hi=127)
    wq = synth.random_packed(N, K, seed=6, stream=7)
    sw = synth.random_scales(N, seed=7)
    srow = synth.random_scales(M, seed=8)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    pq.pq_set_gemm_tile(tile)
    prev = pq.pq_set_gemm_variant(2)
    try:
        out, acc = pq.pq_w4a8_gemm(dev(O.group_even_odd(q)), dev(wq), dev(sw), 0.013, want_out=True, want_acc=True)
        outd, accd = pq.pq_gemm_dynamic(dev(O.group_even_odd(q)), 8, dev(wq), dev(sw), dev(srow), want_out=True,
                                        want_acc=True)
    finally:
        pq.pq_set_gemm_variant(prev)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref) and np.array_equal(host(accd).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.013), sw)).max() <= 1
    assert ulp_diff(host(outd), O.epilogue(acc_ref, srow, sw)).max() <= 1


def test_mixed_width_launch(pq, tile_env):
    """N = 256 a + 192 b with a, b >= 1 and at least 256 tokens: the automatic choice may start tiles of
    two widths in one launch (it does for the benchmark's gate/up shape); small K keeps the oracle fast."""
    pq.pq_set_gemm_tile(-1)
    M, N, K = 2048, 14336, 128
    xq = synth.random_packed(M, K, seed=1)
    wq = synth.random_packed(N, K, seed=2, stream=7)
    sw = synth.random_scales(N, seed=3)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.05, want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.05), sw)).max() <= 1
