"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle.

Gate A (bit-exact): packed codes for unrotated inputs, int32 accumulators, and outputs
within one fp16 ulp of the oracle's epilogue.  Gate B (end to end): pq_linear against the
whole oracle path; codes may differ only at rounding ties (|t - (k + 1/2)| <= 1e-3 code
units, at most 0.1 % of them), the output's max error is at most 1e-2 of max|out|.
"""

import numpy as np
import pytest
import torch

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import check_end_to_end, dev, host, prepare_layer, ulp_diff

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


# ------------------------------------------------------------------ Gate A (i): codes
@pytest.mark.parametrize("M,K,h", [(16, 512, 512), (5, 4096, 4096), (33, 11008, 128), (3, 2048, 128), (7, 8192, 8192)])
def test_codes_exact_on_oracle_rotated_input(pq, M, K, h):
    x = synth.activations(M, K, seed=1)
    sx = O.calibrate_absmax(synth.calibration(K, seed=1), h)
    y16 = O.rotate(x, h).astype(np.float16)
    want = O.pack(O.quantize(y16, sx))
    got = host(pq.pq_rotate_quant(dev(y16), 1, float(sx)))
    assert np.array_equal(got, want)
    got0 = host(pq.pq_rotate_quant(dev(y16), 0, float(sx)))
    assert np.array_equal(got0, want)


@pytest.mark.parametrize("scale", [0.25, 0.1, 0.3, 1.0 / 3.0, 0.7, 0.0123, 1.7, 3e-5, 41.0])
def test_codes_exact_for_every_fp16_value(pq, scale):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    v = bits.view(np.float16)
    v = v[np.isfinite(v)]                       # 63488 finite values
    x = v.reshape(31, 2048)
    s = np.float32(scale)
    got = host(pq.pq_rotate_quant(dev(x), 1, float(s)))
    assert np.array_equal(got, O.pack(O.quantize(x, s)))


def test_codes_exact_at_ties_of_awkward_steps(pq):
    # x = fp16((k + 1/2) * s) for many fp32 steps: quotients sit on or next to a tie
    rng = np.random.default_rng(7)
    for trial in range(6):
        s = np.float32(rng.uniform(0.01, 2.0))
        k = rng.integers(-9, 9, size=(8, 1024)).astype(np.float64)
        x = ((k + 0.5) * np.float64(s)).astype(np.float16)
        got = host(pq.pq_rotate_quant(dev(x), 1, float(s)))
        assert np.array_equal(got, O.pack(O.quantize(x, s))), "step %r" % s


# ------------------------------------------------------------------ Gate A (ii)+(iii): product, epilogue
GEMM_SHAPES = [(16, 512, 512), (1, 512, 512), (3, 48, 96), (4, 4096, 4096), (5, 272, 160), (16, 1024, 11008),
               (17, 512, 512), (31, 48, 32), (33, 272, 4096), (64, 128, 128), (255, 400, 1184), (257, 512, 2048),
               (130, 1040, 14336), (2047, 256, 512)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_product_and_epilogue(pq, M, N, K):
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.2173)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out_ref = O.epilogue(acc_ref, sx, sw)
    for fn in (pq.pq_w4a4_gemm, pq.pq_w4a4_gemm_simple):
        out, acc = fn(dev(xq), dev(wq), dev(sw), float(sx), want_out=True, want_acc=True)
        assert np.array_equal(host(acc).astype(np.int64), acc_ref), fn.__name__
        assert ulp_diff(host(out), out_ref).max() <= 1, fn.__name__
        out2, none = fn(dev(xq), dev(wq), dev(sw), float(sx), want_out=True, want_acc=False)
        assert none is None and np.array_equal(host(out2).view(np.uint16), host(out).view(np.uint16))


@pytest.mark.parametrize("variant,M", [(2, 1), (2, 16), (2, 5), (3, 40), (1, 9), (1, 1), (1, 4), (4, 1), (4, 3), (4, 4), (4, 5), (4, 8), (1, 11), (1, 16)])
def test_forced_variants_agree(pq, variant, M):
    N, K = 256, 1024
    xq, wq = synth.random_packed(M, K, seed=3), synth.random_packed(N, K, seed=4, stream=7)
    sw = synth.random_scales(N, seed=5)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    prev = pq.pq_set_gemm_variant(variant)
    try:
        out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.5, want_out=True, want_acc=True)
    finally:
        pq.pq_set_gemm_variant(prev)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)


@pytest.mark.parametrize("M,N,K", [(6, 4608, 16384), (8, 8192, 28672), (5, 4096, 14336), (7, 256, 32768)])
def test_decode_five_to_eight_tokens_long_rows(pq, M, N, K):
    xq, wq = synth.random_packed(M, K, seed=13), synth.random_packed(N, K, seed=14, stream=7)
    sw = synth.random_scales(N, seed=15)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.25, want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.25), sw)).max() <= 1


@pytest.mark.parametrize("M,N,K", [(1900, 14336, 256), (2048, 14336, 128), (1030, 14336, 384), (2048, 28672, 128), (700, 21504, 128)])
def test_product_mixed_tile_widths(pq, M, N, K):
    """Shapes for which one launch mixes 256- and 192-wide tiles (14336 = 32 x 256 + 32 x 192), ragged in M."""
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.0917)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), float(sx), want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, sx, sw)).max() <= 1
    srow = synth.random_scales(M, seed=M + 3)
    out_d, acc_d = pq.pq_gemm_dynamic(dev(xq), 4, dev(wq), dev(sw), dev(srow), want_out=True, want_acc=True)
    assert np.array_equal(host(acc_d).astype(np.int64), acc_ref)
    assert ulp_diff(host(out_d), O.epilogue(acc_ref, srow, sw)).max() <= 1


def test_product_extreme_codes(pq):
    K = 28672
    for M in (2, 40):
        xq = np.full((M, K // 2), 0x88, np.uint8)          # every code is -8
        wq = np.full((32, K // 2), 0x88, np.uint8)
        wq[16:] = 0x77                                     # and +7 for the second half of the channels
        out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(np.ones(32, np.float32)), 1.0, True, True)
        a = host(acc)
        assert np.all(a[:, :16] == 1835008) and np.all(a[:, 16:] == -56 * K)


# ------------------------------------------------------------------ Gate B: end to end
@pytest.mark.parametrize("M,K,N,h", [(16, 512, 512, 512), (1, 512, 512, 512), (40, 1024, 256, 128),
                                     (70, 4096, 384, 4096), (9, 2048, 256, 1024), (33, 4096, 256, 2048),
                                     (24, 8192, 128, 8192), (4, 16384, 64, 16384), (130, 11008, 256, 128),
                                     (64, 1024, 128, 1), (20, 512, 64, 2), (20, 512, 64, 4), (20, 512, 64, 8),
                                     (20, 512, 64, 16), (20, 512, 64, 32), (20, 512, 64, 64), (20, 512, 64, 256)])
def test_linear_end_to_end(pq, M, K, N, h):
    L = prepare_layer(M, K, N, h, seed=K + h)
    out, ws = pq.pq_linear(dev(L["x"]), dev(L["wq_packed"]), dev(L["sw"]), float(L["sx"]), h)
    xq_gpu = host(ws)[: M * K // 2].reshape(M, K // 2)
    check_end_to_end(L["x"], L["wq_packed"], L["sw"], L["sx"], h, host(out), xq_gpu)


@pytest.mark.parametrize("M,K,N,h", [(1, 4096, 4096, 1), (1, 4096, 6144, 4096), (1, 14336, 4096, 128), (2, 14336, 512, 128),
                                     (3, 8192, 256, 8192), (4, 4096, 1024, 1), (4, 2048, 128, 1024), (1, 11008, 256, 128),
                                     (4, 28672, 64, 128), (1, 28672, 8192, 128), (2, 1024, 48, 2048 // 2), (1, 32, 16, 32),
                                     (3, 96, 32, 1), (1, 8192, 10240, 1),
                                     # rows quantized from the registers they were loaded into: all four pieces of a
                                     # thread, a partial last piece, rotation blocks of 64 to 512 channels
                                     (4, 8192, 256, 1), (3, 10240, 64, 1), (2, 8192, 128, 512), (1, 2048, 64, 256),
                                     (4, 4096, 64, 64), (2, 12288, 32, 128)])
def test_decode_fused_linear(pq, M, K, N, h):
    # M <= 4: pq_linear is one fused launch; codes in the workspace, output against the oracle
    L = prepare_layer(M, K, N, h, seed=K + N + h)
    for variant in (0, 4):      # automatic choice, and the fused launch forced wherever it is supported
        prev = pq.pq_set_gemm_variant(variant)
        try:
            out, ws = pq.pq_linear(dev(L["x"]), dev(L["wq_packed"]), dev(L["sw"]), float(L["sx"]), h)
        finally:
            pq.pq_set_gemm_variant(prev)
        xq_gpu = host(ws)[: M * K // 2].reshape(M, K // 2)
        check_end_to_end(L["x"], L["wq_packed"], L["sw"], L["sx"], h, host(out), xq_gpu)
        if h <= 1:      # unrotated: codes are exact
            assert np.array_equal(xq_gpu, O.pack(O.quantize(L["x"], L["sx"])))


def test_rotation_involution_on_device(pq):
    # H is its own inverse up to h: rotating the dequantised rotation gives x back within the step
    K, h = 4096, 4096
    x = synth.activations(8, K, seed=5)
    s = np.float32(2.0 ** -9)                    # fine step: every code saturates, so use a coarse check
    y = O.rotate(x, h)
    s = np.float32(np.abs(y).max() / 7)
    q = O.unpack(host(pq.pq_rotate_quant(dev(x), h, float(s))))
    assert np.abs(q.astype(np.float64) * s - y).max() <= 0.5 * s * (1 + 1e-3)


def test_deterministic(pq):
    L = prepare_layer(48, 4096, 512, 4096, seed=2)
    args = (dev(L["x"]), dev(L["wq_packed"]), dev(L["sw"]), float(L["sx"]), 4096)
    o1, w1 = pq.pq_linear(*args)
    o2, w2 = pq.pq_linear(*args)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(w1, w2)


def test_runs_on_side_stream(pq):
    L = prepare_layer(32, 512, 128, 128, seed=4)
    st = torch.cuda.Stream()
    a = [dev(L["x"]), dev(L["wq_packed"]), dev(L["sw"])]
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        out, ws = pq.pq_linear(a[0], a[1], a[2], float(L["sx"]), 128)
    st.synchronize()
    ref = O.linear(L["x"], L["wq_packed"], L["sw"], L["sx"], 128)
    assert np.max(np.abs(host(out).astype(np.float64) - ref.astype(np.float64))) <= 1e-2 * np.abs(ref).max()
