"""The calls under HIP graph capture: captured once, replayed several times with new contents in
the same buffers and eager work in between; every replay must give the eager result bit for bit.
(The library enqueues kernels only: no allocation, no memset, no synchronisation, so every call
can be captured.  The benchmark times its decode legs this way.)"""

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


@pytest.mark.parametrize("M,K,N,h,planes", [(1, 4096, 4096, 1, False), (1, 14336, 512, 128, False),
                                            (4, 4096, 1024, 1, False), (16, 4096, 2048, 1, False),
                                            (12, 14336, 512, 128, False), (24, 4096, 1024, 1, False),
                                            (300, 1024, 768, 128, False), (48, 14336, 1024, 128, True),
                                            (100, 4096, 2048, 1, True)])
def test_linear_replays_match_eager(pq, M, K, N, h, planes):
    """planes: the workspace also holds the partial sums of the split-K launch (two more kernels in the graph)."""
    wq, sw = O.weight_rtn(synth.weights(N, K, seed=3))
    wp = dev(O.pack(wq))
    dsw = dev(sw)
    xs = [synth.activations(M, K, seed=40 + i) for i in range(3)]
    sx = float(O.calibrate_absmax(synth.calibration(K, 3), h))
    x = dev(xs[0])
    out = torch.empty((M, N), dtype=torch.float16, device="cuda")
    nbytes = pq.pq_linear_workspace_bytes_split(M, N, K) if planes else pq.pq_linear_workspace_bytes(M, K)
    assert not planes or nbytes > pq.pq_linear_workspace_bytes(M, K)
    work = torch.empty((max(256, nbytes),), dtype=torch.uint8, device="cuda")
    eager = []
    for xi in xs:
        x.copy_(torch.from_numpy(xi))
        o, _ = pq.pq_linear(x, wp, dsw, sx, h)
        eager.append(host(o).view(np.uint16).copy())
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        x.copy_(torch.from_numpy(xs[0]))
        pq.pq_linear(x, wp, dsw, sx, h, out=out, workspace=work)          # warm-up on the capture stream
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            pq.pq_linear(x, wp, dsw, sx, h, out=out, workspace=work)
    torch.cuda.synchronize()
    for rep in range(2):
        for i, xi in enumerate(xs):
            x.copy_(torch.from_numpy(xi))
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(host(out).view(np.uint16), eager[i]), (rep, i)
            # eager work of the same library between replays
            pq.pq_rotate_quant(x, h, sx)
            torch.cuda.synchronize()


@pytest.mark.parametrize("M,K,N,h", [(300, 1024, 768, 128), (256, 512, 896, 1), (130, 2048, 512, 512), (64, 4096, 256, 4096)])
def test_prepacked_linear_replays_match_eager(pq, M, K, N, h):
    """pq_linear_f6 (tile-writing quantizer or matrix-pipe rotation, persistent product kernel, N = 896 as two tile
    widths in one launch, the 4096-point rotation through quantizer + repack) captured and replayed."""
    wq, sw = O.weight_rtn(synth.weights(N, K, seed=5))
    w6 = pq.pq_repack_f6(dev(O.pack(wq)))
    dsw = dev(sw)
    xs = [synth.activations(M, K, seed=60 + i) for i in range(3)]
    sx = float(O.calibrate_absmax(synth.calibration(K, 5), h))
    x = dev(xs[0])
    out = torch.empty((M, N), dtype=torch.float16, device="cuda")
    work = torch.empty((max(256, pq.pq_linear_f6_workspace_bytes(M, K, h)),), dtype=torch.uint8, device="cuda")
    eager = []
    for xi in xs:
        x.copy_(torch.from_numpy(xi))
        o, _ = pq.pq_linear_f6(x, w6, dsw, sx, h)
        eager.append(host(o).view(np.uint16).copy())
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        x.copy_(torch.from_numpy(xs[0]))
        pq.pq_linear_f6(x, w6, dsw, sx, h, out=out, workspace=work)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            pq.pq_linear_f6(x, w6, dsw, sx, h, out=out, workspace=work)
    torch.cuda.synchronize()
    for rep in range(2):
        for i, xi in enumerate(xs):
            x.copy_(torch.from_numpy(xi))
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(host(out).view(np.uint16), eager[i]), (rep, i)
            pq.pq_rotate_quant_f6(x, h if h <= 512 else 1, sx)            # eager work of the same library between replays
            torch.cuda.synchronize()


def test_two_matrices_replay_matches_eager(pq):
    """pq_linear2 at one token (one fused launch for both matrices) and at 40 tokens (quantizer + two products)."""
    K, Na, Nb, h = 4096, 1024, 528, 1
    wa, swa = O.weight_rtn(synth.weights(Na, K, seed=7))
    wb, swb = O.weight_rtn(synth.weights(Nb, K, seed=8))
    dwa, dswa, dwb, dswb = dev(O.pack(wa)), dev(swa), dev(O.pack(wb)), dev(swb)
    sx = float(O.calibrate_absmax(synth.calibration(K, 7), h))
    for M in (1, 40):
        xs = [synth.activations(M, K, seed=70 + i) for i in range(2)]
        x = dev(xs[0])
        oa = torch.empty((M, Na), dtype=torch.float16, device="cuda")
        ob = torch.empty((M, Nb), dtype=torch.float16, device="cuda")
        work = torch.empty((max(256, pq.pq_linear_workspace_bytes(M, K)),), dtype=torch.uint8, device="cuda")
        eager = []
        for xi in xs:
            x.copy_(torch.from_numpy(xi))
            a, b, _ = pq.pq_linear2(x, dwa, dswa, dwb, dswb, sx, h)
            eager.append((host(a).view(np.uint16).copy(), host(b).view(np.uint16).copy()))
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            pq.pq_linear2(x, dwa, dswa, dwb, dswb, sx, h, out_a=oa, out_b=ob, workspace=work)
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                pq.pq_linear2(x, dwa, dswa, dwb, dswb, sx, h, out_a=oa, out_b=ob, workspace=work)
        torch.cuda.synchronize()
        for rep in range(2):
            for i, xi in enumerate(xs):
                x.copy_(torch.from_numpy(xi))
                oa.zero_(); ob.zero_()
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert np.array_equal(host(oa).view(np.uint16), eager[i][0]) and np.array_equal(host(ob).view(np.uint16), eager[i][1]), (M, rep, i)


def test_quantizer_family_replays_match_eager(pq):
    M, K = 64, 4096
    xs = [synth.activations(M, K, seed=50 + i) for i in range(3)]
    x = dev(xs[0])
    q4 = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    q8 = torch.empty((M, K), dtype=torch.int8, device="cuda")
    qd = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    srow = torch.empty((M,), dtype=torch.float32, device="cuda")
    eager = []
    for xi in xs:
        x.copy_(torch.from_numpy(xi))
        a = pq.pq_rotate_quant(x, 128, 0.4)
        b = pq.pq_rotate_quant8(x, 128, 0.02)
        c, s = pq.pq_rotate_quant_dynamic(x, 128, 1.0, 4)
        eager.append((host(a).copy(), host(b).copy(), host(c).copy(), host(s).copy()))
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        pq.pq_rotate_quant(x, 128, 0.4, out=q4)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            pq.pq_rotate_quant(x, 128, 0.4, out=q4)
            pq.pq_rotate_quant8(x, 128, 0.02, out=q8)
            pq.pq_rotate_quant_dynamic(x, 128, 1.0, 4, out=qd, row_scale=srow)
    torch.cuda.synchronize()
    for rep in range(2):
        for i, xi in enumerate(xs):
            x.copy_(torch.from_numpy(xi))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            a, b, c, s = eager[i]
            assert np.array_equal(host(q4), a) and np.array_equal(host(q8), b)
            assert np.array_equal(host(qd), c) and np.array_equal(host(srow), s)


def test_two_streams_at_once(pq):
    """The library keeps no state between calls: different layers on two streams at the same time."""
    cases = []
    for seed, (M, K, N, h) in enumerate([(16, 4096, 4096, 1), (2048, 1024, 1024, 128)]):
        wq, sw = O.weight_rtn(synth.weights(N, K, seed=seed))
        x = dev(synth.activations(M, K, seed=60 + seed))
        sx = float(O.calibrate_absmax(synth.calibration(K, seed), h))
        wp, dsw = dev(O.pack(wq)), dev(sw)
        ref, _ = pq.pq_linear(x, wp, dsw, sx, h)
        cases.append((x, wp, dsw, sx, h, host(ref).view(np.uint16).copy(), torch.cuda.Stream(),
                      torch.empty((M, N), dtype=torch.float16, device="cuda"),
                      torch.empty((max(256, pq.pq_linear_workspace_bytes(M, K)),), dtype=torch.uint8, device="cuda")))
    torch.cuda.synchronize()
    for rep in range(20):
        for x, wp, dsw, sx, h, ref, st, out, work in cases:
            with torch.cuda.stream(st):
                pq.pq_linear(x, wp, dsw, sx, h, out=out, workspace=work)
    torch.cuda.synchronize()
    for x, wp, dsw, sx, h, ref, st, out, work in cases:
        assert np.array_equal(host(out).view(np.uint16), ref)


def test_roofline_probes_run(pq):
    """The two measuring sticks of the benchmark: they must run, read in bounds and leave their sink alone."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    ops = pq.pq_probe_mfma_i8(torch.zeros(4096, dtype=torch.int8, device="cuda"), 10, 256, sink)
    assert ops == 256 * 4 * 10 * 16 * 65536
    ops = pq.pq_probe_mfma_i8(torch.full((16,), 0x70, dtype=torch.int8, device="cuda"), 3, 7, sink)   # one operand set, reused
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    assert pq.pq_probe_stream_read(src, sink) == 4 << 20
    assert pq.pq_probe_stream_read(src[:4 * 37], sink) == 16 * 37                                    # shorter than one pass
    torch.cuda.synchronize()
    assert int(sink.abs().sum().item()) == 0
