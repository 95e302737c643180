"""GPU parity of the split-K launch of the tiled product (pq_w4a4_gemm_ws, some dozens to some
hundreds of tokens) against the oracle.

Integer work: the accumulators are bit-exact whatever the number of K runs, and the fp16 outputs are
bit-identical to the unsplit tiled kernel's (the reduce kernel applies the same expression).  Shapes
cover: the three tile heights, token counts that are no multiple of a tile, output widths that are no
multiple of 128, run counts that do not divide the number of 128-channel stages, a K with the
minimum of two stages per run, a workspace that is too small (fewer planes, or none), a workspace
larger than asked for, the automatic choice at the sizes of the benchmark's linears, and pq_linear
with the planes behind its codes.
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


def forced(pq, variant, fn, *a, **kw):
    prev = pq.pq_set_gemm_variant(variant)
    try:
        return fn(*a, **kw)
    finally:
        pq.pq_set_gemm_variant(prev)


def scratch(nbytes, fill=0xA5):
    import torch
    return torch.full((max(int(nbytes), 256),), fill, dtype=torch.uint8, device="cuda")


# (tokens, channels out, channels in): forced split, up to 5 runs
SHAPES = [(33, 256, 512), (100, 384, 1024), (128, 1024, 4096), (129, 272, 1280), (200, 528, 2048), (257, 256, 1024),
          (64, 144, 14336), (300, 1040, 1664), (48, 16, 640)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_forced_split_product_and_epilogue(pq, M, N, K):
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.2173)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    nbytes = forced(pq, 5, pq.pq_w4a4_gemm_workspace_bytes, M, N, K)
    runs = min(5, K // 256)
    assert nbytes == runs * M * N * 4
    ws = scratch(nbytes)
    out, acc = forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), float(sx), ws, want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, sx, sw)).max() <= 1
    tiled, _ = forced(pq, 2, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), float(sx))
    assert np.array_equal(host(tiled).view(np.uint16), host(out).view(np.uint16))
    # each output alone
    only_out, none = forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), float(sx), ws, want_out=True)
    assert none is None and np.array_equal(host(only_out).view(np.uint16), host(out).view(np.uint16))
    none, only_acc = forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), float(sx), ws, want_out=False,
                            want_acc=True)
    assert none is None and np.array_equal(host(only_acc), host(acc))


def test_extreme_codes_do_not_overflow(pq):
    """All codes -8: every partial plane holds the largest sums the format allows."""
    M, N, K = 40, 64, 8192
    xq = np.full((M, K // 2), 0x88, dtype=np.uint8)
    wq = np.full((N, K // 2), 0x88, dtype=np.uint8)
    sw = synth.random_scales(N, seed=1)
    ws = scratch(5 * M * N * 4)
    out, acc = forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), 0.01, ws, want_out=True, want_acc=True)
    assert (host(acc) == 64 * K).all()
    assert ulp_diff(host(out), O.epilogue(np.full((M, N), 64 * K, dtype=np.int64), np.float32(0.01), sw)).max() <= 1


def test_small_and_large_workspaces(pq):
    M, N, K = 96, 256, 2048
    xq = synth.random_packed(M, K, seed=3)
    wq = synth.random_packed(N, K, seed=4, stream=7)
    sw = synth.random_scales(N, seed=5)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    plane = M * N * 4
    for nbytes in (5 * plane + 4096, 3 * plane, 2 * plane + 100):     # 5, 3 and 2 runs
        ws = scratch(nbytes)
        _, acc = forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), 0.1, ws, want_out=False, want_acc=True)
        assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    # the part of a larger workspace beyond the planes is left alone
    ws = scratch(5 * plane + 4096, fill=0x5A)
    forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), 0.1, ws, want_out=True)
    assert (host(ws)[5 * plane:] == 0x5A).all()
    # no two planes: the forced variant refuses, the automatic choice runs unsplit
    with pytest.raises(RuntimeError, match="PQ_ERR_UNSUPPORTED"):
        forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), 0.1, scratch(plane), want_out=True)
    with pytest.raises(RuntimeError, match="PQ_ERR_UNSUPPORTED"):
        forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), 0.1, None, want_out=True)
    _, acc = pq.pq_w4a4_gemm_ws(dev(xq), dev(wq), dev(sw), 0.1, scratch(plane), want_out=False, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    _, acc = pq.pq_w4a4_gemm_ws(dev(xq), dev(wq), dev(sw), 0.1, None, want_out=False, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)


def test_short_k_cannot_split(pq):
    M, N, K = 64, 128, 384          # three stages: no two runs of two
    assert forced(pq, 5, pq.pq_w4a4_gemm_workspace_bytes, M, N, K) == 0
    xq = synth.random_packed(M, K, seed=3)
    wq = synth.random_packed(N, K, seed=4, stream=7)
    sw = synth.random_scales(N, seed=5)
    with pytest.raises(RuntimeError, match="PQ_ERR_UNSUPPORTED"):
        forced(pq, 5, pq.pq_w4a4_gemm_ws, dev(xq), dev(wq), dev(sw), 0.1, scratch(1 << 20), want_out=True)
    # K no multiple of 128: the ragged kernel, never split
    assert pq.pq_w4a4_gemm_workspace_bytes(64, 4096, 14336 + 32) == 0


def test_misaligned_workspace_is_refused(pq):
    M, N, K = 64, 128, 1024
    xq = synth.random_packed(M, K, seed=3)
    wq = synth.random_packed(N, K, seed=4, stream=7)
    sw = synth.random_scales(N, seed=5)
    ws = scratch(1 << 20)
    with pytest.raises(RuntimeError, match="PQ_ERR_ALIGN"):
        pq.pq_w4a4_gemm_ws(dev(xq), dev(wq), dev(sw), 0.1, ws[16:], want_out=True)


@pytest.mark.parametrize("M,N,K", [(64, 4096, 14336), (24, 4096, 14336), (40, 4096, 4096), (64, 6144, 4096),
                                   (256, 4096, 14336), (24, 14336, 4096)])
def test_automatic_choice_at_benchmark_shapes(pq, M, N, K):
    """The cost model splits these (the workspace query says so); sampled outputs against the oracle,
    everything against the unsplit kernel."""
    nbytes = pq.pq_w4a4_gemm_workspace_bytes(M, N, K)
    assert nbytes >= 2 * M * N * 4 and nbytes % (M * N * 4) == 0
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    out, acc = pq.pq_w4a4_gemm_ws(dev(xq), dev(wq), dev(sw), 0.11, scratch(nbytes), want_out=True, want_acc=True)
    ref_out, ref_acc = forced(pq, 2, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), 0.11, want_out=True, want_acc=True)
    assert np.array_equal(host(acc), host(ref_acc))
    assert np.array_equal(host(out).view(np.uint16), host(ref_out).view(np.uint16))
    rng = np.random.default_rng(M + N)
    rows, cols = rng.integers(0, M, 8), rng.integers(0, N, 64)
    sub = O.gemm_i64(O.unpack(xq[rows]), O.unpack(wq[cols]))
    assert np.array_equal(host(acc)[np.ix_(rows, cols)].astype(np.int64), sub)


def test_no_planes_asked_for_where_nothing_splits(pq):
    for M, N, K in [(1, 4096, 4096), (16, 4096, 14336), (2048, 4096, 14336), (2048, 14336, 4096), (0, 4096, 4096)]:
        assert pq.pq_w4a4_gemm_workspace_bytes(M, N, K) == 0
    assert pq.pq_linear_workspace_bytes_split(2048, 4096, 14336) == pq.pq_linear_workspace_bytes(2048, 14336)


@pytest.mark.parametrize("M,N,K,h", [(64, 4096, 14336, 128), (100, 1024, 4096, 4096), (24, 4096, 14336, 128)])
def test_linear_with_planes_behind_the_codes(pq, M, N, K, h):
    x = synth.activations(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = 0.21
    small = pq.pq_linear_workspace_bytes(M, K)
    full = pq.pq_linear_workspace_bytes_split(M, N, K)
    assert full > small
    ref, codes_ref = pq.pq_linear(dev(x), dev(wq), dev(sw), sx, h, workspace=scratch(small))
    out, ws = pq.pq_linear(dev(x), dev(wq), dev(sw), sx, h, workspace=scratch(full))
    assert np.array_equal(host(out).view(np.uint16), host(ref).view(np.uint16))
    assert np.array_equal(host(ws)[:M * K // 2], host(codes_ref)[:M * K // 2])
    # and the layer against the oracle, from the codes the library wrote
    codes = host(ws)[:M * K // 2].reshape(M, K // 2)
    acc_ref = O.gemm_i64(O.unpack(codes), O.unpack(wq))
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(sx), sw)).max() <= 1


# ---------------------------------------------------------------- the widened products, split
WIDE_SHAPES = [(33, 256, 512), (100, 384, 1024), (129, 272, 1280), (257, 256, 1024), (64, 144, 14336), (48, 16, 640)]


@pytest.mark.parametrize("M,N,K", WIDE_SHAPES)
def test_forced_split_int8_activations(pq, M, N, K):
    q = synth.random_codes(M, K, seed=M + K, stream=9, lo=-128, hi=127)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.0173)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    xq8 = O.group_even_odd(q)
    nbytes = forced(pq, 5, pq.pq_gemm_workspace_bytes, M, N, K, 8)
    assert nbytes == min(5, K // 256) * M * N * 4
    out, acc = forced(pq, 5, pq.pq_w4a8_gemm_ws, dev(xq8), dev(wq), dev(sw), float(sx), scratch(nbytes),
                      want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, sx, sw)).max() <= 1
    tiled, _ = forced(pq, 2, pq.pq_w4a8_gemm, dev(xq8), dev(wq), dev(sw), float(sx))
    assert np.array_equal(host(tiled).view(np.uint16), host(out).view(np.uint16))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("M,N,K", WIDE_SHAPES)
def test_forced_split_per_token_steps(pq, bits, M, N, K):
    lo, hi = (-128, 127) if bits == 8 else (-8, 7)
    q = synth.random_codes(M, K, seed=M + K, stream=9, lo=lo, hi=hi)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    srow = synth.random_scales(M, seed=M + 1)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    xq = O.group_even_odd(q) if bits == 8 else O.pack(q)
    ws = scratch(forced(pq, 5, pq.pq_gemm_workspace_bytes, M, N, K, bits))
    out, acc = forced(pq, 5, pq.pq_gemm_dynamic_ws, dev(xq), bits, dev(wq), dev(sw), dev(srow), ws,
                      want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, srow, sw)).max() <= 1
    tiled, _ = forced(pq, 2, pq.pq_gemm_dynamic, dev(xq), bits, dev(wq), dev(sw), dev(srow))
    assert np.array_equal(host(tiled).view(np.uint16), host(out).view(np.uint16))


@pytest.mark.parametrize("M,N,K,z", [(33, 256, 512, 3), (100, 384, 1024, 0), (129, 272, 1280, 15), (64, 144, 14336, 6),
                                     (40, 64, 32768, 11)])
def test_forced_split_zero_point(pq, M, N, K, z):
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.173)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    corr = (8 - z) * O.unpack(wq).astype(np.int64).sum(axis=1)
    d_corr = pq.pq_zero_point_correction(dev(wq), z)
    ws = scratch(forced(pq, 5, pq.pq_gemm_workspace_bytes, M, N, K, 4))
    out, acc = forced(pq, 5, pq.pq_w4a4_gemm_zp_ws, dev(xq), dev(wq), dev(sw), float(sx), d_corr, ws,
                      want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)          # raw accumulators, without the correction
    assert ulp_diff(host(out), O.epilogue(acc_ref + corr[None, :], sx, sw)).max() <= 1
    tiled, _ = forced(pq, 2, pq.pq_w4a4_gemm_zp, dev(xq), dev(wq), dev(sw), float(sx), d_corr)
    assert np.array_equal(host(tiled).view(np.uint16), host(out).view(np.uint16))


def test_widened_layers_with_planes_behind_their_workspace(pq):
    M, N, K, h = 64, 4096, 14336, 128
    x = synth.activations(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    small, full = pq.pq_linear_w4a8_workspace_bytes(M, K), pq.pq_linear_w4a8_workspace_bytes_split(M, N, K)
    assert full > small
    ref, _ = pq.pq_linear_w4a8(dev(x), dev(wq), dev(sw), 0.021, h, workspace=scratch(small))
    out, ws = pq.pq_linear_w4a8(dev(x), dev(wq), dev(sw), 0.021, h, workspace=scratch(full))
    assert np.array_equal(host(out).view(np.uint16), host(ref).view(np.uint16))
    acc_ref = O.gemm_i64(O.ungroup_even_odd(host(ws)[:M * K].view(np.int8).reshape(M, K)), O.unpack(wq))
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.021), sw)).max() <= 1
    for bits in (4, 8):
        small = pq.pq_linear_dynamic_workspace_bytes(M, K, bits)
        full = pq.pq_linear_dynamic_workspace_bytes_split(M, N, K, bits)
        assert full > small
        ref, _ = pq.pq_linear_dynamic(dev(x), dev(wq), dev(sw), h, bits=bits, workspace=scratch(small))
        out, _ = pq.pq_linear_dynamic(dev(x), dev(wq), dev(sw), h, bits=bits, workspace=scratch(full))
        assert np.array_equal(host(out).view(np.uint16), host(ref).view(np.uint16))


def test_random_shapes_split_equals_unsplit(pq):
    """Seeded random shapes through the automatic choice with a generous workspace: whatever the cost
    model picks (tile height, number of runs, or no split at all), accumulators and outputs equal the
    unsplit tiled kernel's; small cases also against the oracle."""
    rng = np.random.default_rng(20241005)
    ws = scratch(96 << 20)
    split = 0
    for case in range(48):
        M = int(rng.integers(17, 420))
        N = 16 * int(rng.integers(1, 300))
        K = 128 * int(rng.integers(1, 90))
        xq = synth.random_packed(M, K, seed=case)
        wq = synth.random_packed(N, K, seed=case, stream=7)
        sw = synth.random_scales(N, seed=case)
        split += pq.pq_w4a4_gemm_workspace_bytes(M, N, K) > 0
        out, acc = pq.pq_w4a4_gemm_ws(dev(xq), dev(wq), dev(sw), 0.07, ws, want_out=True, want_acc=True)
        ref_out, ref_acc = forced(pq, 2, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), 0.07, want_out=True, want_acc=True)
        assert np.array_equal(host(acc), host(ref_acc)), (M, N, K)
        assert np.array_equal(host(out).view(np.uint16), host(ref_out).view(np.uint16)), (M, N, K)
        if M * N * K <= 3e8:
            assert np.array_equal(host(acc).astype(np.int64), O.gemm_i64(O.unpack(xq), O.unpack(wq))), (M, N, K)
    assert split >= 12          # the draw exercises the split launch, not only the fallback


def test_random_shapes_widened_products_with_planes(pq):
    """Seeded random shapes through the automatic choice of the int8, per-token and zero-point
    products with a generous workspace, against the oracle."""
    rng = np.random.default_rng(5265)
    ws = scratch(64 << 20)
    for case in range(30):
        M = int(rng.integers(9, 300))
        N = 16 * int(rng.integers(1, 120))
        K = 128 * int(rng.integers(1, 40))
        q = synth.random_codes(M, K, seed=case, stream=9, lo=-128, hi=127)
        xq = synth.random_packed(M, K, seed=case)
        wq = synth.random_packed(N, K, seed=case, stream=7)
        sw = synth.random_scales(N, seed=case)
        srow = synth.random_scales(M, seed=case + 1)
        a8 = O.gemm_i64(q, O.unpack(wq))
        a4 = O.gemm_i64(O.unpack(xq), O.unpack(wq))
        out, acc = pq.pq_w4a8_gemm_ws(dev(O.group_even_odd(q)), dev(wq), dev(sw), 0.013, ws, want_out=True, want_acc=True)
        assert np.array_equal(host(acc).astype(np.int64), a8), (M, N, K)
        assert ulp_diff(host(out), O.epilogue(a8, np.float32(0.013), sw)).max() <= 1, (M, N, K)
        out, acc = pq.pq_gemm_dynamic_ws(dev(xq), 4, dev(wq), dev(sw), dev(srow), ws, want_out=True, want_acc=True)
        assert np.array_equal(host(acc).astype(np.int64), a4), (M, N, K)
        assert ulp_diff(host(out), O.epilogue(a4, srow, sw)).max() <= 1, (M, N, K)
        z = int(rng.integers(0, 16))
        corr = (8 - z) * O.unpack(wq).astype(np.int64).sum(axis=1)
        out, acc = pq.pq_w4a4_gemm_zp_ws(dev(xq), dev(wq), dev(sw), 0.07, pq.pq_zero_point_correction(dev(wq), z), ws,
                                         want_out=True, want_acc=True)
        assert np.array_equal(host(acc).astype(np.int64), a4), (M, N, K)
        assert ulp_diff(host(out), O.epilogue(a4 + corr[None, :], np.float32(0.07), sw)).max() <= 1, (M, N, K, z)
