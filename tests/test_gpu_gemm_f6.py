"""GPU parity of the product on the 6-bit floating-point matrix instruction (pq_repack_f6 +
pq_w4a4_gemm_f6) against the oracle.

The repacked layout is checked byte for byte against a plain numpy construction written from its
definition in the header (E3M2 code of every value, 32 values of 6 bits per lane as a little-endian bit
stream of 24 bytes, 64 lanes x 2 steps per block of 32 rows x 128 channels stored as four planes, blocks
ordered [row block][group]).  The product's
accumulators are the oracle's integer sums bit for bit (fp32 accumulation of such operands is exact),
the outputs within 1 ulp of the oracle's epilogue and bit-identical to the INT8 tiled kernel's.
"""

import os

import numpy as np
import pytest
import torch

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import dev, host, ulp_diff

pytestmark = pytest.mark.gpu

E3M2 = np.array([0, 12, 16, 18, 20, 21, 22, 23, 24], dtype=np.uint64)     # codes of 0..8: exponent bias 3, 2 mantissa bits


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


def tiles_by_definition(q):
    """q: int8 codes [R, K] -> the repacked bytes, from the layout's definition."""
    R, K = q.shape
    RB, KS = (R + 31) // 32, K // 64
    qp = np.zeros((RB * 32, K), np.int64)
    qp[:R] = q
    enc = E3M2[np.abs(qp)] | (np.uint64(32) * (qp < 0).astype(np.uint64))
    # [rb][row in block][group][step][half][i] -> [group][rb][half][row in block][step][i]
    # (lane = 32 half + row in block; a lane's two images, first step then second, lie side by side)
    v = enc.reshape(RB, 32, KS // 2, 2, 2, 32).transpose(2, 0, 4, 1, 3, 5).reshape(-1, 32)
    words = np.zeros((v.shape[0], 3), dtype=np.uint64)
    for i in range(32):
        bit = 6 * i
        words[:, bit // 64] |= v[:, i] << np.uint64(bit % 64)
        if bit % 64 > 58:
            words[:, bit // 64 + 1] |= v[:, i] >> np.uint64(64 - bit % 64)
    # a block of 32 rows x 128 channels: 64 lanes x 2 steps x 24 bytes, stored as four planes, each lane after
    # lane: bytes 0-15 of the first step's images, their bytes 16-23, bytes 0-7 of the second step's, their
    # bytes 8-23
    img = words.view(np.uint8).reshape(-1, 64, 2, 24)
    planes = [img[:, :, 0, :16], img[:, :, 0, 16:], img[:, :, 1, :8], img[:, :, 1, 8:]]
    return np.concatenate([p.reshape(img.shape[0], -1) for p in planes], axis=1).reshape(-1)


@pytest.mark.parametrize("R,K", [(32, 128), (33, 256), (100, 1152), (256, 4096), (1, 128)])
def test_repacked_layout_matches_its_definition(pq, R, K):
    q = synth.random_codes(R, K, seed=R + K)
    got = host(pq.pq_repack_f6(dev(O.pack(q))))
    want = tiles_by_definition(q)
    assert pq.pq_f6_tiles_bytes(R, K) == want.size
    assert np.array_equal(got[:want.size], want)


@pytest.fixture
def tile_env(pq):
    saved = pq.pq_set_gemm_f6_tile(-1)
    yield
    pq.pq_set_gemm_f6_tile(saved)


@pytest.mark.parametrize("tile", ["auto", "2", "4"])     # channels per tile: by shape, 128, 256
@pytest.mark.parametrize("M,N,K", [(256, 256, 128), (256, 256, 512), (300, 400, 1152), (64, 128, 128), (517, 784, 384),
                                   (129, 1040, 2048), (1, 16, 128), (2048, 512, 256), (40, 4096, 4096)])
def test_product_and_epilogue(pq, tile_env, tile, M, N, K):
    pq.pq_set_gemm_f6_tile(-1 if tile == "auto" else int(tile))
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.0917)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    x6, w6 = pq.pq_repack_f6(dev(xq)), pq.pq_repack_f6(dev(wq))
    out, acc = pq.pq_w4a4_gemm_f6(x6, w6, dev(sw), float(sx), M, N, K, want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, sx, sw)).max() <= 1
    prev = pq.pq_set_gemm_variant(2)
    try:
        tiled, _ = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), float(sx))
    finally:
        pq.pq_set_gemm_variant(prev)
    assert np.array_equal(host(tiled).view(np.uint16), host(out).view(np.uint16))
    only_out, none = pq.pq_w4a4_gemm_f6(x6, w6, dev(sw), float(sx), M, N, K, want_out=True)
    assert none is None and np.array_equal(host(only_out).view(np.uint16), host(out).view(np.uint16))


def test_extreme_codes_on_a_long_row(pq):
    M, N, K = 40, 48, 65536
    xq = np.full((M, K // 2), 0x88, np.uint8)          # every code -8
    wq = np.full((N, K // 2), 0x88, np.uint8)
    sw = synth.random_scales(N, seed=1)
    out, acc = pq.pq_w4a4_gemm_f6(pq.pq_repack_f6(dev(xq)), pq.pq_repack_f6(dev(wq)), dev(sw), 0.01, M, N, K,
                                  want_out=True, want_acc=True)
    assert (host(acc) == 64 * K).all()
    assert ulp_diff(host(out), O.epilogue(np.full((M, N), 64 * K, np.int64), np.float32(0.01), sw)).max() <= 1


def test_benchmark_shape_sampled(pq):
    M, N, K = 2048, 4096, 4096
    xq = synth.random_packed(M, K, seed=11)
    wq = synth.random_packed(N, K, seed=12, stream=7)
    sw = synth.random_scales(N, seed=13)
    _, acc = pq.pq_w4a4_gemm_f6(pq.pq_repack_f6(dev(xq)), pq.pq_repack_f6(dev(wq)), dev(sw), 0.1, M, N, K,
                                want_out=False, want_acc=True)
    rng = np.random.default_rng(5)
    rows, cols = rng.integers(0, M, 32), rng.integers(0, N, 256)
    sub = O.gemm_i64(O.unpack(xq[rows]), O.unpack(wq[cols]))
    assert np.array_equal(host(acc)[np.ix_(rows, cols)].astype(np.int64), sub)
    prev = pq.pq_set_gemm_variant(2)
    try:
        _, ref = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.1, want_out=False, want_acc=True)
    finally:
        pq.pq_set_gemm_variant(prev)
    assert np.array_equal(host(acc), host(ref))


def test_argument_errors(pq):
    x6 = pq.pq_repack_f6(dev(synth.random_packed(32, 128, seed=1)))
    w6 = pq.pq_repack_f6(dev(synth.random_packed(16, 128, seed=2)))
    sw = dev(synth.random_scales(16, seed=3))
    with pytest.raises(pq.PQError, match="PQ_ERR_SHAPE"):
        pq.pq_repack_f6(dev(np.zeros((32, 32), np.uint8)))              # K = 64
    with pytest.raises(pq.PQError, match="PQ_ERR_SCALE"):
        pq.pq_w4a4_gemm_f6(x6, w6, sw, 0.0, 32, 16, 128)
    with pytest.raises(pq.PQError, match="PQ_ERR_NULL"):
        pq.pq_w4a4_gemm_f6(x6, w6, sw, 0.1, 32, 16, 128, want_out=False, want_acc=False)


def codes_of_tiles(tiles, R, K):
    """Inverse of tiles_by_definition: the int8 codes [R, K] behind a repacked byte stream."""
    RB, KS = (R + 31) // 32, K // 64
    blocks = np.asarray(tiles[:RB * (KS // 2) * 3072]).reshape(-1, 3072)
    img = np.zeros((blocks.shape[0], 64, 2, 24), np.uint8)
    img[:, :, 0, :16] = blocks[:, :1024].reshape(-1, 64, 16)
    img[:, :, 0, 16:] = blocks[:, 1024:1536].reshape(-1, 64, 8)
    img[:, :, 1, :8] = blocks[:, 1536:2048].reshape(-1, 64, 8)
    img[:, :, 1, 8:] = blocks[:, 2048:].reshape(-1, 64, 16)
    bits = np.unpackbits(img.reshape(-1, 24), axis=1, bitorder="little").reshape(-1, 32, 6)
    e = (bits * (1 << np.arange(6))).sum(axis=2)                      # 6-bit values, little-endian stream
    mag = np.full(64, -99, np.int64)
    mag[E3M2.astype(np.int64)] = np.arange(9)
    val = np.where(e >= 32, -mag[e & 31], mag[e & 31])
    assert (mag[e & 31] >= 0).all()
    # [group][rb][half][row in block][step][i] -> [rb][row in block][group][step][half][i]
    v = val.reshape(KS // 2, RB, 2, 32, 2, 32).transpose(1, 3, 0, 4, 2, 5).reshape(RB * 32, K)
    assert not v[R:].any()
    return v[:R].astype(np.int8)


def test_codes_of_tiles_inverts_the_definition():
    q = synth.random_codes(45, 384, seed=3)
    assert np.array_equal(codes_of_tiles(tiles_by_definition(q), 45, 384), q)


@pytest.mark.parametrize("M,K,N,h", [(300, 1152, 400, 1), (2048, 4096, 512, 1), (33, 128, 16, 0), (70, 14336, 512, 128),
                                     (256, 4096, 1024, 4096), (1, 256, 64, 1), (100, 1536, 64, 512), (65, 2048, 32, 2048)])
def test_layer_with_prepacked_weights(pq, M, K, N, h):
    """pq_linear_f6 against pq_linear: the same codes and the same outputs bit for bit; the tiles it leaves are
    the repacked codes (rotation blocks beyond 512 channels: the canonical codes lie behind them); and (through
    pq_linear's own parity) the oracle."""
    x = synth.activations(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = 0.213
    ref, ref_ws = pq.pq_linear(dev(x), dev(wq), dev(sw), sx, h)
    ref_codes = host(ref_ws)[:M * K // 2].reshape(M, K // 2)
    w6 = pq.pq_repack_f6(dev(wq))
    out, ws = pq.pq_linear_f6(dev(x), w6, dev(sw), sx, h)
    assert np.array_equal(host(out).view(np.uint16), host(ref).view(np.uint16))
    tiles_bytes = pq.pq_f6_tiles_bytes(M, K)
    off = (tiles_bytes + 255) // 256 * 256
    assert pq.pq_linear_f6_workspace_bytes(M, K, h) == off + (M * K // 2 + 255) // 256 * 256 * (h > 512)
    assert np.array_equal(host(ws)[:tiles_bytes], tiles_by_definition(O.unpack(ref_codes)))
    assert np.array_equal(codes_of_tiles(host(ws), M, K), O.unpack(ref_codes))
    if h > 512:
        assert np.array_equal(host(ws)[off:off + M * K // 2].reshape(M, K // 2), ref_codes)
    acc_ref = O.gemm_i64(O.unpack(ref_codes), O.unpack(wq))
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(sx), sw)).max() <= 1


@pytest.mark.parametrize("M,K,h", [(70, 1152, 1), (33, 512, 128), (300, 4096, 512), (2048, 14336, 128)])
def test_tile_writing_quantizer(pq, M, K, h):
    """pq_rotate_quant_f6: the tiles are those of pq_rotate_quant's codes, with and without the canonical copy."""
    x = synth.activations(M, K, seed=M + K + h)
    sx = 0.187
    codes = host(pq.pq_rotate_quant(dev(x), h, sx))
    want = tiles_by_definition(O.unpack(codes))
    nib = torch.full((M, K // 2), 0xAA, dtype=torch.uint8, device="cuda")
    both = pq.pq_rotate_quant_f6(dev(x), h, sx, codes=nib)
    assert np.array_equal(host(both)[:want.size], want) and np.array_equal(host(nib), codes)
    assert np.array_equal(host(pq.pq_rotate_quant_f6(dev(x), h, sx))[:want.size], want)
    with pytest.raises(pq.PQError, match="PQ_ERR_UNSUPPORTED"):
        pq.pq_rotate_quant_f6(dev(synth.activations(4, 2048, seed=1)), 1024, sx)


@pytest.mark.parametrize("M,K", [(1, 128), (37, 640), (100, 1408), (32, 512), (65, 14336), (21900, 1152)])
def test_rotation_of_128_point_blocks_on_the_matrix_pipe(pq, M, K):
    """128-point blocks take the kernel that rotates with matrix instructions (both outputs of it: canonical
    nibbles and tiles).  Against the oracle's fp64 rotation: codes differ only where the rotated value is at a
    rounding tie; token counts that are not multiples of 32, channel counts that are not multiples of 512.
    The last case is large enough (6165 blocks) for the launch in which a wavefront takes two blocks, with an
    odd number of blocks per row (the last wavefront of a row has one)."""
    x = synth.activations(M, K, seed=3 * M + K)
    y = O.rotate(x, 128)
    sx = np.float32(np.abs(y).max() / 7.0)
    want = O.quantize(y, sx)
    codes = host(pq.pq_rotate_quant(dev(x), 128, float(sx)))
    nib = torch.full((M, K // 2), 0x55, dtype=torch.uint8, device="cuda")
    tiles = pq.pq_rotate_quant_f6(dev(x), 128, float(sx), codes=nib)
    assert np.array_equal(host(nib), codes)
    assert np.array_equal(codes_of_tiles(host(tiles), M, K), O.unpack(codes))
    assert np.array_equal(host(tiles)[: pq.pq_f6_tiles_bytes(M, K)], tiles_by_definition(O.unpack(codes)))
    got = O.unpack(codes).astype(np.int32)
    diff = got - want.astype(np.int32)
    at = np.nonzero(diff)
    assert at[0].size <= 1e-3 * diff.size
    if at[0].size:
        assert np.all(np.abs(diff[at]) == 1)
        t = y[at] / np.float64(sx)
        assert np.all(np.abs(t - (np.minimum(got[at], want[at]) + 0.5)) <= 1e-3)


def test_outputs_larger_than_the_l2s(pq):
    """A launch whose codes or images exceed 32 MiB writes them with ordinary stores, a smaller one streams them
    out: same bytes either way.  17000 x 4096 unrotated: 34.8 MB of nibbles, 52 MB of images; codes against the
    oracle's (exact without rotation), images against the layout's definition."""
    M, K = 17000, 4096
    x = synth.activations(M, K, seed=21)
    sx = np.float32(0.21)
    want = O.pack(O.quantize(x, sx))
    codes = host(pq.pq_rotate_quant(dev(x), 0, float(sx)))
    assert np.array_equal(codes, want)
    nib = torch.full((M, K // 2), 0x33, dtype=torch.uint8, device="cuda")
    tiles = host(pq.pq_rotate_quant_f6(dev(x), 0, float(sx), codes=nib))
    assert np.array_equal(host(nib), want)
    del nib
    assert np.array_equal(tiles[: pq.pq_f6_tiles_bytes(M, K)], tiles_by_definition(O.unpack(want)))


def test_rotation_on_the_matrix_pipe_one_hot_and_constant_rows(pq):
    """Rows whose rotation is known in closed form: a one-hot row becomes +-v / sqrt(128) in its block (the signs
    are a row of the Hadamard matrix), a constant block becomes sqrt(128) v in its first channel and zero elsewhere."""
    K = 384
    x = np.zeros((130, K), dtype=np.float16)
    for r in range(128):
        x[r, 128 + r] = np.float16(3.0 + (r % 5))            # one-hot at every position of the second block
    x[128, :128] = np.float16(0.25)                           # constant first block
    x[129, 256:] = np.float16(-1.5)                           # constant third block
    sx = np.float32(0.1)                                      # 3..7 / sqrt(128) / 0.1 = 2.65 .. 6.19: away from ties
    want = O.quantize(O.rotate(x, 128), sx)
    got = O.unpack(host(pq.pq_rotate_quant(dev(x), 128, float(sx))))
    assert np.array_equal(got, want)
    assert np.array_equal(codes_of_tiles(host(pq.pq_rotate_quant_f6(dev(x), 128, float(sx))), 130, K), want)


def test_prepack_names(pq):
    """pq_prepacked_bytes / pq_prepack_weights / pq_linear_prepacked are the tile calls under their other names."""
    M, K, N, h = 70, 1152, 272, 128
    x = synth.activations(M, K, seed=9)
    wq, sw = O.weight_rtn(synth.weights(N, K, seed=9))
    dw, dsw = dev(O.pack(wq)), dev(sw)
    assert pq.pq_prepacked_bytes(N, K) == pq.pq_f6_tiles_bytes(N, K)
    tiled = pq.pq_prepack_weights(dw)
    assert torch.equal(tiled, pq.pq_repack_f6(dw))
    a, _ = pq.pq_linear_prepacked(dev(x), tiled, dsw, 0.21, h)
    b, _ = pq.pq_linear_f6(dev(x), tiled, dsw, 0.21, h)
    c, _ = pq.pq_linear(dev(x), dw, dsw, 0.21, h)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(a.view(torch.int16), c.view(torch.int16))


def test_unrotated_quantizer_to_tiles_is_exact_for_every_fp16_value(pq):
    """The tile-writing quantizer (no rotation) on all finite fp16 values and on constructed ties: the codes
    behind the tiles equal the oracle's."""
    v = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    x = v[np.isfinite(v)].reshape(31, 2048)
    for s in (0.25, 1.0 / 3.0, 0.0123, 41.0):
        tiles = pq.pq_rotate_quant_f6(dev(x), 1, s)
        assert np.array_equal(codes_of_tiles(host(tiles), 31, 2048), O.quantize(x, np.float32(s))), s
    rng = np.random.default_rng(17)
    s = np.float32(0.0371)
    k = rng.integers(-10, 10, size=(8, 1024)).astype(np.float64)
    xt = ((k + 0.5) * np.float64(s)).astype(np.float16)
    tiles = pq.pq_rotate_quant_f6(dev(xt), 0, float(s))
    assert np.array_equal(codes_of_tiles(host(tiles), 8, 1024), O.quantize(xt, s))


@pytest.mark.parametrize("M,N,K", [(300, 448, 256), (40, 4096, 1152), (517, 1216, 384), (2048, 14336, 128)])
def test_mixed_width_launch(pq, tile_env, M, N, K):
    """N = 256 a + 192 b: tiles of both widths in one launch (forced; the automatic choice takes it for the
    benchmark's gate/up shape, the last case)."""
    pq.pq_set_gemm_f6_tile(-1 if (M, N) == (2048, 14336) else 3)
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out, acc = pq.pq_w4a4_gemm_f6(pq.pq_repack_f6(dev(xq)), pq.pq_repack_f6(dev(wq)), dev(sw), 0.0917, M, N, K,
                                  want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.0917), sw)).max() <= 1
