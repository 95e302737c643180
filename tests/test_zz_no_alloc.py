"""pq_linear_noalloc (the layer with the library's built-in scratch array, for callers that cannot
allocate) against pq_linear with a caller's workspace: outputs equal bit for bit, on calls in a row
that share the array, each smaller than the one before, through the tiled, the matrix-streaming
and the fused decode kernels; sizes beyond the array are refused with nothing enqueued.
"""

import numpy as np
import pytest
import torch

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import check_end_to_end, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


def _layer(M, K, N, h, seed):
    x = synth.activations(M, K, seed)
    wq, sw = O.weight_rtn(synth.weights(N, K, seed))
    sx = O.calibrate_absmax(synth.calibration(K, seed), h)
    return x, O.pack(wq), sw, sx


# (M, K, N, h): prefill tiles with a ragged token tail; a serving batch (planes behind the codes);
# 16 tokens on streamed matrix tiles; one token in the fused launch
SEQUENCE = [(389, 2048, 1280, 128), (40, 4096, 1024, 4096), (16, 1024, 512, 1), (1, 1024, 768, 128)]


def test_noalloc_equals_pq_linear_on_calls_in_a_row(pq):
    prepared = []
    for i, (M, K, N, h) in enumerate(SEQUENCE):
        x, wq_packed, sw, sx = _layer(M, K, N, h, seed=40 + i)
        d = {"x": dev(x), "wq": dev(wq_packed), "sw": dev(sw), "sx": float(sx), "h": h,
             "out": torch.empty((M, N), dtype=torch.float16, device="cuda"), "host": (x, wq_packed, sw, sx)}
        d["ref"], d["ref_ws"] = pq.pq_linear(d["x"], d["wq"], d["sw"], d["sx"], h)
        prepared.append(d)
    torch.cuda.synchronize()
    # the calls share the array: back to back on one stream, outputs read only at the end
    for d in prepared:
        d["out"].fill_(float("nan"))
        pq.pq_linear_noalloc(d["x"], d["wq"], d["sw"], d["sx"], d["h"], d["out"])
    torch.cuda.synchronize()
    for d, (M, K, N, h) in zip(prepared, SEQUENCE):
        got, ref = host(d["out"]), host(d["ref"])
        assert np.array_equal(got.view(np.uint16), ref.view(np.uint16)), (M, K, N, h)
    # and the existing entry point is itself right on the largest and the smallest of them (gate B)
    for d, (M, K, N, h) in ((prepared[0], SEQUENCE[0]), (prepared[-1], SEQUENCE[-1])):
        x, wq_packed, sw, sx = d["host"]
        xq = host(d["ref_ws"])[: M * K // 2].reshape(M, K // 2)
        check_end_to_end(x, wq_packed, sw, sx, h, host(d["out"]), xq)


def test_noalloc_second_pass_in_reverse_order(pq):
    # the array now holds the last call's contents: growing sizes must not see them either
    for i, (M, K, N, h) in reversed(list(enumerate(SEQUENCE))):
        x, wq_packed, sw, sx = _layer(M, K, N, h, seed=40 + i)
        dx, dw, ds = dev(x), dev(wq_packed), dev(sw)
        ref, _ = pq.pq_linear(dx, dw, ds, float(sx), h)
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        pq.pq_linear_noalloc(dx, dw, ds, float(sx), h, out)
        torch.cuda.synchronize()
        assert np.array_equal(host(out).view(np.uint16), host(ref).view(np.uint16)), (M, K, N, h)


def test_noalloc_limits(pq):
    L = pq.lib()
    limit = pq.pq_linear_noalloc_max_bytes()
    assert limit == 32 << 20
    x = torch.zeros((8, 64), dtype=torch.float16, device="cuda")
    w = torch.zeros((16, 32), dtype=torch.uint8, device="cuda")
    s = torch.ones((16,), dtype=torch.float32, device="cuda")
    o = torch.zeros((8, 16), dtype=torch.float16, device="cuda")
    args = lambda M, K: (x.data_ptr(), w.data_ptr(), s.data_ptr(), 1.0, 1, M, 16, K, o.data_ptr(), None)
    # codes beyond the array: refused before anything looks at the buffers
    assert L.pq_linear_noalloc(*args(2048, 2 * (limit // 2048) + 64)) == pq.PQ_ERR_WORKSPACE
    assert L.pq_linear_noalloc(*args(1 << 40, 64)) == pq.PQ_ERR_WORKSPACE
    assert L.pq_linear_noalloc(*args(4, 1 << 40)) == pq.PQ_ERR_WORKSPACE
    # other argument errors are pq_linear's
    assert L.pq_linear_noalloc(*args(8, 48)) == pq.PQ_ERR_SHAPE
    assert L.pq_linear_noalloc(x.data_ptr(), None, s.data_ptr(), 1.0, 1, 8, 16, 64, o.data_ptr(), None) == pq.PQ_ERR_NULL
    assert L.pq_linear_noalloc(*args(0, 64)) == pq.PQ_OK
    # exactly at the limit the size check passes (2048 tokens of 32768 channels; not launched here: the
    # buffers above are tiny, so only the host-side answer for a NULL input is taken)
    assert L.pq_linear_noalloc(None, w.data_ptr(), s.data_ptr(), 1.0, 1, 2048, 16, 32768, o.data_ptr(), None) == pq.PQ_ERR_NULL
    torch.cuda.synchronize()
