"""GPU parity of pq_linear2 (two weight matrices on the same tokens, gate and up of an MLP block).

Against the oracle: the layer's gate of the other tests (codes differ from the oracle's only at rounding ties,
the oracle's product and epilogue on the GPU's codes reproduce both outputs within one fp16 ulp).  Against
pq_linear: outputs bit-identical to two separate calls, in the fused single launch (few tokens; one row
group may start in the first matrix and the next in the second, matrices of different heights, with and
without rotation) and in the quantize-once + two products form (more tokens).
"""

import numpy as np
import pytest

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import check_end_to_end, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


def layer(M, K, Na, Nb, h, seed):
    x = synth.activations(M, K, seed)
    sx = O.calibrate_absmax(synth.calibration(K, seed), h)
    wa, swa = O.weight_rtn(synth.weights(Na, K, seed))
    wb, swb = O.weight_rtn(synth.weights(Nb, K, seed + 1))
    return x, sx, O.pack(wa), swa, O.pack(wb), swb


# (M, K, N_a, N_b, had_block): one token to a small prefill; heights that make 1, 2 or 4 rows per wavefront;
# N_a not a multiple of the rows a workgroup takes at a time; 5 tokens and 64 tokens leave the fused launch
CASES = [(1, 512, 256, 256, 1), (1, 4096, 1008, 528, 1), (2, 2048, 4096, 2064, 128), (4, 1024, 16, 8192, 64),
         (1, 8192, 14336, 14336, 1), (3, 4096, 9008, 9008, 4096), (1, 14336, 2048, 1040, 128),
         (1, 4096, 14336, 14336, 1),      # gate and up of Llama-3-8B at one token: the launch bench.py times

         (5, 1024, 528, 272, 128), (64, 1024, 528, 272, 1), (16, 4096, 1024, 512, 128)]


@pytest.mark.parametrize("M,K,Na,Nb,h", CASES)
def test_two_matrices_one_quantization(pq, M, K, Na, Nb, h):
    x, sx, wa, swa, wb, swb = layer(M, K, Na, Nb, h, seed=M + K + Na)
    dx, dwa, dswa, dwb, dswb = dev(x), dev(wa), dev(swa), dev(wb), dev(swb)
    oa, ob, ws = pq.pq_linear2(dx, dwa, dswa, dwb, dswb, float(sx), h)
    codes = host(ws)[: M * K // 2].reshape(M, K // 2)
    check_end_to_end(x, wa, swa, sx, h, host(oa), codes)
    check_end_to_end(x, wb, swb, sx, h, host(ob), codes)
    ra, _ = pq.pq_linear(dx, dwa, dswa, float(sx), h)
    rb, wsb = pq.pq_linear(dx, dwb, dswb, float(sx), h)
    assert np.array_equal(host(oa).view(np.uint16), host(ra).view(np.uint16))
    assert np.array_equal(host(ob).view(np.uint16), host(rb).view(np.uint16))
    assert np.array_equal(codes, host(wsb)[: M * K // 2].reshape(M, K // 2))


@pytest.mark.parametrize("M,K,Na,Nb,h", [(70, 1152, 272, 528, 128), (300, 512, 896, 256, 1), (33, 4096, 64, 512, 4096)])
def test_two_matrices_prepacked(pq, M, K, Na, Nb, h):
    """pq_linear2_f6: the outputs of two pq_linear_f6 calls, and of pq_linear2 on the canonical weights, bit for bit."""
    x, sx, wa, swa, wb, swb = layer(M, K, Na, Nb, h, seed=M + K)
    dx, dwa, dswa, dwb, dswb = dev(x), dev(wa), dev(swa), dev(wb), dev(swb)
    ta, tb = pq.pq_repack_f6(dwa), pq.pq_repack_f6(dwb)
    oa, ob, _ = pq.pq_linear2_f6(dx, ta, dswa, tb, dswb, float(sx), h)
    ra, _ = pq.pq_linear_f6(dx, ta, dswa, float(sx), h)
    rb, _ = pq.pq_linear_f6(dx, tb, dswb, float(sx), h)
    ca, cb, _ = pq.pq_linear2(dx, dwa, dswa, dwb, dswb, float(sx), h)
    for got, one, canon in ((oa, ra, ca), (ob, rb, cb)):
        assert np.array_equal(host(got).view(np.uint16), host(one).view(np.uint16))
        assert np.array_equal(host(got).view(np.uint16), host(canon).view(np.uint16))


def test_argument_errors(pq):
    import torch
    x, sx, wa, swa, wb, swb = layer(1, 512, 32, 32, 1, seed=3)
    dx, dwa, dswa, dwb, dswb = dev(x), dev(wa), dev(swa), dev(wb), dev(swb)
    with pytest.raises(Exception):
        pq.pq_linear2(dx, dwa, dswa, dwb[:24], dswb[:24], float(sx), 1)          # N_b not a multiple of 16
    with pytest.raises(Exception):
        pq.pq_linear2(dx, dwa, dswa, dwb, dswb, float(sx), 1, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    with pytest.raises(Exception):
        pq.pq_linear2(dx, dwa, dswa, dwb, dswb, 0.0, 1)
