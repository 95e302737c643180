"""GPU parity of the weight-streaming matrix-tile kernel (2..16 tokens of given codes) against the oracle.

Integer work: accumulators are bit-exact.  Outputs are within one fp16 ulp of the oracle's epilogue
(the kernel rounds the product of the integer sum and the fp32 step to fp32, then to fp16), and
bit-identical to the tiled kernel's, so that a row's output does not depend on how many tokens are
in the batch.  Shapes cover: one and several row groups per workgroup task (short and long K),
ragged numbers of row groups, slices of K that do not divide evenly (K = 11008), workgroups with
more tasks than partial-sum tiles (the tiles are cleared and reused), every token count, int8
activations, per-token steps and the zero-point correction of Eq. 1.
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


SHAPES = [(16, 512, 256), (9, 272, 512), (16, 4096, 4096), (13, 1040, 14336), (16, 6144, 4096), (2, 48, 768),
          (11, 4112, 11008), (16, 14336, 4096), (7, 4096, 14336), (4, 256, 32768), (4, 16, 65536), (1, 528, 2048)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_matrix_tiles_product_and_epilogue(pq, M, N, K):
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.2173)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out, acc = forced(pq, 1, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), float(sx), want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, sx, sw)).max() <= 1
    tiled, _ = forced(pq, 2, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), float(sx))
    assert np.array_equal(host(tiled).view(np.uint16), host(out).view(np.uint16))
    only_out, none = forced(pq, 1, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), float(sx), want_out=True, want_acc=False)
    assert none is None and np.array_equal(host(only_out).view(np.uint16), host(out).view(np.uint16))


@pytest.mark.parametrize("M", list(range(1, 17)))
def test_every_token_count(pq, M):
    N, K = 4800, 4096            # 300 row groups: 44 workgroups take two of them, the others one
    xq = synth.random_packed(M, K, seed=100 + M)
    wq = synth.random_packed(N, K, seed=7, stream=7)
    sw = synth.random_scales(N, seed=2)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.31, want_out=True, want_acc=True)   # automatic choice
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.31), sw)).max() <= 1
    out1, acc1 = forced(pq, 1, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), 0.31, want_out=True, want_acc=True)
    assert np.array_equal(host(acc1), host(acc))
    assert np.array_equal(host(out1).view(np.uint16), host(out).view(np.uint16))


@pytest.mark.parametrize("M,N,K", [(3, 66128, 256), (16, 131072 + 48, 512), (9, 70000 - 70000 % 16, 1024)])
def test_more_tasks_than_sum_tiles(pq, M, N, K):
    """Short rows and very many of them: a workgroup runs through more tasks than it has
    partial-sum tiles, so the tiles are cleared and reused behind a barrier."""
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    out, acc = forced(pq, 1, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), 0.05, want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.05), sw)).max() <= 1


def test_extreme_codes_longest_row(pq):
    for a, w in ((-8, -8), (7, -8), (-8, 7), (7, 7)):
        M, N, K = 4, 32, 65536
        xq = O.pack(np.full((M, K), a, np.int8))
        wq = O.pack(np.full((N, K), w, np.int8))
        sw = np.full(N, 2.0 ** -14, np.float32)
        out, acc = forced(pq, 1, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), 1.0, want_out=True, want_acc=True)
        assert np.all(host(acc) == a * w * K)
        assert ulp_diff(host(out), O.epilogue(np.full((M, N), a * w * K, np.int64), np.float32(1), sw)).max() <= 1


@pytest.mark.parametrize("M,N,K", [(16, 512, 256), (9, 272, 1024), (16, 4096, 4096), (8, 4096, 14336), (5, 1040, 11008),
                                   (12, 6144, 8192), (3, 14336, 4096), (16, 64, 8192)])
def test_int8_activations(pq, M, N, K):
    q = synth.random_codes(M, K, seed=M + K, stream=9, lo=-128, hi=127)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    xq8 = O.group_even_odd(q)
    out, acc = forced(pq, 1, pq.pq_w4a8_gemm, dev(xq8), dev(wq), dev(sw), 0.02, want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.02), sw)).max() <= 1
    auto, acc0 = pq.pq_w4a8_gemm(dev(xq8), dev(wq), dev(sw), 0.02, want_out=True, want_acc=True)
    assert np.array_equal(host(acc0), host(acc))
    assert np.array_equal(host(auto).view(np.uint16), host(out).view(np.uint16))


def test_int8_extreme_codes(pq):
    for a, w in ((-128, -8), (127, -8), (-128, 7)):
        M, N, K = 8, 32, 16384
        q = np.full((M, K), a, np.int8)
        wq = O.pack(np.full((N, K), w, np.int8))
        sw = np.full(N, 2.0 ** -18, np.float32)
        out, acc = forced(pq, 1, pq.pq_w4a8_gemm, dev(O.group_even_odd(q)), dev(wq), dev(sw), 1.0, want_out=True,
                          want_acc=True)
        assert np.all(host(acc) == a * w * K)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("M,N,K", [(16, 512, 512), (9, 1040, 4096), (12, 4096, 14336), (6, 272, 8192)])
def test_per_token_steps(pq, bits, M, N, K):
    if bits == 8 and M * (K // 16 + 16) * 16 > 140 * 1024:
        M = 8                                            # int8 codes of 12 tokens x 14336 do not fit in LDS
    lo, hi = (-128, 127) if bits == 8 else (-8, 7)
    q = synth.random_codes(M, K, seed=M + K, stream=9, lo=lo, hi=hi)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    srow = synth.random_scales(M, seed=M + 1)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    xq = O.group_even_odd(q) if bits == 8 else O.pack(q)
    out, acc = forced(pq, 1, pq.pq_gemm_dynamic, dev(xq), bits, dev(wq), dev(sw), dev(srow), want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, srow, sw)).max() <= 1
    tiled, _ = forced(pq, 2, pq.pq_gemm_dynamic, dev(xq), bits, dev(wq), dev(sw), dev(srow))
    assert np.array_equal(host(tiled).view(np.uint16), host(out).view(np.uint16))


@pytest.mark.parametrize("M,N,K,z", [(16, 512, 512, 3), (9, 272, 1024, 15), (12, 4096, 14336, 6), (5, 6144, 8192, 0)])
def test_zero_point_correction_in_the_epilogue(pq, M, N, K, z):
    xq = synth.random_packed(M, K, seed=M + K)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    sx = np.float32(0.173)
    acc_ref = O.gemm_i64(O.unpack(xq), O.unpack(wq))
    corr = (8 - z) * O.unpack(wq).astype(np.int64).sum(axis=1)
    d_corr = pq.pq_zero_point_correction(dev(wq), z)
    out, acc = forced(pq, 1, pq.pq_w4a4_gemm_zp, dev(xq), dev(wq), dev(sw), float(sx), d_corr, want_out=True,
                      want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref + corr[None, :], sx, sw)).max() <= 1


def test_kernels_agree_bit_for_bit(pq):
    """The same row gives the same fp16 output whichever kernel the token count selects."""
    N, K = 2048, 4096
    xq = synth.random_packed(16, K, seed=21)
    wq = synth.random_packed(N, K, seed=22, stream=7)
    sw = synth.random_scales(N, seed=23)
    ref, _ = forced(pq, 2, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), 0.1)
    ref = host(ref).view(np.uint16)
    for M in (1, 2, 4, 5, 8, 9, 16):
        out, _ = pq.pq_w4a4_gemm(dev(xq[:M]), dev(wq), dev(sw), 0.1)
        assert np.array_equal(host(out).view(np.uint16), ref[:M]), M
    simple, _ = pq.pq_w4a4_gemm_simple(dev(xq), dev(wq), dev(sw), 0.1)
    assert np.array_equal(host(simple).view(np.uint16), ref)


def test_unsupported_shapes_are_refused_when_forced(pq):
    xq = synth.random_packed(4, 384, seed=1)
    wq = synth.random_packed(64, 384, seed=2, stream=7)
    sw = synth.random_scales(64, seed=3)
    with pytest.raises(pq.PQError) as e:                 # K is not a multiple of 256
        forced(pq, 1, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), 0.1)
    assert e.value.status == 7
    out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.1, want_out=True, want_acc=True)   # automatic: another kernel
    assert np.array_equal(host(acc).astype(np.int64), O.gemm_i64(O.unpack(xq), O.unpack(wq)))


def test_random_shapes(pq):
    """Seeded random shapes within the kernel's limits: every combination of slices per row group,
    ring depth, ragged row groups and token count that the fixed cases above may have missed."""
    rng = np.random.default_rng(20241005)
    for case in range(40):
        bits = 8 if case % 3 == 2 else 4
        K = 256 * int(rng.integers(1, 49))
        N = 16 * int(rng.integers(1, max(2, min(1500, 30_000_000 // K // 16))))
        M = int(rng.integers(1, 17))
        while not 16448 + M * ((K if bits == 8 else K // 2) + 16) <= 160 * 1024:
            M -= 1
        lo, hi = (-128, 127) if bits == 8 else (-8, 7)
        q = synth.random_codes(M, K, seed=case, stream=9, lo=lo, hi=hi)
        wq = synth.random_packed(N, K, seed=case, stream=7)
        sw = synth.random_scales(N, seed=case)
        acc_ref = O.gemm_i64(q, O.unpack(wq))
        if bits == 8:
            out, acc = forced(pq, 1, pq.pq_w4a8_gemm, dev(O.group_even_odd(q)), dev(wq), dev(sw), 0.07, want_out=True,
                              want_acc=True)
        else:
            out, acc = forced(pq, 1, pq.pq_w4a4_gemm, dev(O.pack(q)), dev(wq), dev(sw), 0.07, want_out=True, want_acc=True)
        assert np.array_equal(host(acc).astype(np.int64), acc_ref), (case, bits, M, N, K)
        assert ulp_diff(host(out), O.epilogue(acc_ref, np.float32(0.07), sw)).max() <= 1, (case, bits, M, N, K)


@pytest.mark.parametrize("bits,M,N,K", [(4, 16, 272, 32768), (4, 11, 8192, 28672), (8, 16, 528, 14336), (8, 9, 64, 16384)])
def test_tokens_split_over_two_launches(pq, bits, M, N, K):
    """The codes of all tokens do not fit in LDS together: the call runs the first half of the
    tokens, then the rest (pointer offsets into codes, steps, accumulators and outputs)."""
    lo, hi = (-128, 127) if bits == 8 else (-8, 7)
    q = synth.random_codes(M, K, seed=M + K, stream=9, lo=lo, hi=hi)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    srow = synth.random_scales(M, seed=M + 3)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    xq = O.group_even_odd(q) if bits == 8 else O.pack(q)
    out, acc = forced(pq, 1, pq.pq_gemm_dynamic, dev(xq), bits, dev(wq), dev(sw), dev(srow), want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, srow, sw)).max() <= 1
    if bits == 8:
        out2, acc2 = pq.pq_w4a8_gemm(dev(xq), dev(wq), dev(sw), 0.04, want_out=True, want_acc=True)       # automatic choice
    else:
        out2, acc2 = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.04, want_out=True, want_acc=True)
    assert np.array_equal(host(acc2).astype(np.int64), acc_ref)
    assert ulp_diff(host(out2), O.epilogue(acc_ref, np.float32(0.04), sw)).max() <= 1


def test_codes_of_half_the_tokens_must_fit(pq):
    xq = synth.random_packed(16, 65536, seed=1)
    wq = synth.random_packed(32, 65536, seed=2, stream=7)
    sw = synth.random_scales(32, seed=3)
    with pytest.raises(pq.PQError) as e:
        forced(pq, 1, pq.pq_w4a4_gemm, dev(xq), dev(wq), dev(sw), 0.1)
    assert e.value.status == 7
    out, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq), dev(sw), 0.1, want_out=True, want_acc=True)   # automatic: the tiled kernel
    assert np.array_equal(host(acc).astype(np.int64), O.gemm_i64(O.unpack(xq), O.unpack(wq)))


@pytest.mark.parametrize("bits,M,N,K", [(4, 17, 512, 512), (4, 32, 4096, 4096), (4, 24, 4096, 14336), (4, 29, 272, 28672),
                                        (8, 32, 1040, 4096), (8, 20, 528, 14336)])
def test_seventeen_to_thirty_two_tokens(pq, bits, M, N, K):
    """Blocks of 16 tokens in consecutive launches (and halves of a block whose codes do not fit)."""
    lo, hi = (-128, 127) if bits == 8 else (-8, 7)
    q = synth.random_codes(M, K, seed=M + K, stream=9, lo=lo, hi=hi)
    wq = synth.random_packed(N, K, seed=N + K, stream=7)
    sw = synth.random_scales(N, seed=N)
    srow = synth.random_scales(M, seed=M + 5)
    acc_ref = O.gemm_i64(q, O.unpack(wq))
    xq = O.group_even_odd(q) if bits == 8 else O.pack(q)
    out, acc = forced(pq, 1, pq.pq_gemm_dynamic, dev(xq), bits, dev(wq), dev(sw), dev(srow), want_out=True, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(host(out), O.epilogue(acc_ref, srow, sw)).max() <= 1
    tiled, _ = forced(pq, 2, pq.pq_gemm_dynamic, dev(xq), bits, dev(wq), dev(sw), dev(srow))
    assert np.array_equal(host(tiled).view(np.uint16), host(out).view(np.uint16))
    fn = pq.pq_w4a8_gemm if bits == 8 else pq.pq_w4a4_gemm
    auto, acc0 = fn(dev(xq), dev(wq), dev(sw), 0.03, want_out=True, want_acc=True)          # automatic choice
    assert np.array_equal(host(acc0).astype(np.int64), acc_ref)
    assert ulp_diff(host(auto), O.epilogue(acc_ref, np.float32(0.03), sw)).max() <= 1
