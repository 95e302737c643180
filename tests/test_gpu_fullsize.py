"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run whole Llama-sized layers in seconds, so rows are sampled: tokens are
independent, hence the oracle's result for a sampled token is its result inside the full
batch.  Codes and int32 accumulators of the sampled tokens must be exact (gate A); the
fp16 outputs of the whole layer call must pass the end-to-end gate on those tokens (gate B).
Both forms of the layer run: the canonical one against the oracle, the prepacked one (the
benchmark's headline) against the canonical one, every output and accumulator bit for bit.
"""

import numpy as np
import pytest
import torch

import oracle as O
from paper_2410_05265_amd import synth
from pq_testlib import check_end_to_end, dev, host, ulp_diff

pytestmark = pytest.mark.gpu

# name -> (K, N, online Hadamard block as in bench.py)
L3_8B = [("qkv", 4096, 6144, 1), ("o", 4096, 4096, 1), ("gate", 4096, 14336, 1), ("down", 14336, 4096, 128)]


@pytest.fixture(scope="module")
def pq():
    import paper_2410_05265_amd.binding as b
    b.lib()
    return b


_weights_cache = {}


def _weights(N, K, seed):
    """Packed RTN weights of a layer; the last few are kept (the 70B matrices take ~15 s to draw and round)."""
    key = (N, K, seed)
    if key not in _weights_cache:
        while len(_weights_cache) >= 2:
            _weights_cache.pop(next(iter(_weights_cache)))
        wq, sw = O.weight_rtn(synth.weights(N, K, seed))
        _weights_cache[key] = (O.pack(wq), sw)
    return _weights_cache[key]


def _layer(M, K, N, h, seed):
    x = synth.activations(M, K, seed)
    wq_packed, sw = _weights(N, K, seed)
    sx = O.calibrate_absmax(synth.calibration(K, seed), h)
    return x, wq_packed, sw, sx


def _check_sampled(pq, M, K, N, h, seed, nsample):
    x, wq_packed, sw, sx = _layer(M, K, N, h, seed)
    rng = np.random.default_rng(seed + 1000)
    rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, size=nsample)]))
    d_w, d_sw = dev(wq_packed), dev(sw)
    out, ws = pq.pq_linear(dev(x), d_w, d_sw, float(sx), h)
    xq_all = ws[: M * K // 2].view(M, K // 2)
    # the same launch configuration with raw accumulators (verification output)
    _, acc = pq.pq_w4a4_gemm(xq_all.contiguous(), d_w, d_sw, float(sx), want_out=False, want_acc=True)
    torch.cuda.synchronize()
    # the prepacked form of the same layer (what bench.py times as its headline): the whole output and all
    # accumulators bit-identical to the canonical form's, so the gates below hold for both
    if K % 128 == 0:
        w6 = pq.pq_repack_f6(d_w)
        out6, ws6 = pq.pq_linear_f6(dev(x), w6, d_sw, float(sx), h)
        assert torch.equal(out6.view(torch.int16), out.view(torch.int16)), "pq_linear_f6 differs from pq_linear"
        _, acc6 = pq.pq_w4a4_gemm_f6(ws6, w6, d_sw, float(sx), M, N, K, want_out=False, want_acc=True)
        assert torch.equal(acc6, acc), "accumulators of the 6-bit product differ"
        del w6, out6, ws6, acc6
    xq_s, out_s, acc_s = host(xq_all[rows]), host(out[rows]), host(acc[rows])
    del out, ws, acc
    # gate A on the sampled tokens: accumulators exact for the GPU's own codes
    acc_ref = O.gemm_i64(O.unpack(xq_s), O.unpack(wq_packed))
    assert np.array_equal(acc_s.astype(np.int64), acc_ref)
    if h <= 1:
        assert np.array_equal(xq_s, O.pack(O.quantize(x[rows], sx)))
    # gate B on the sampled tokens
    check_end_to_end(x[rows], wq_packed, sw, sx, h, out_s, xq_s)


@pytest.mark.parametrize("name,K,N,h", L3_8B)
def test_llama3_8b_prefill_2048(pq, name, K, N, h):
    _check_sampled(pq, 2048, K, N, h, seed=11, nsample=24)


def test_llama3_8b_prefill_2048_down_every_token(pq):
    """The headline shape un-sampled: all 2048 x 4096 accumulators of down_proj against the oracle's int64
    product of the GPU's own codes, and every fp16 output within one ulp of the oracle's epilogue."""
    M, K, N, h = 2048, 14336, 4096, 128
    x, wq_packed, sw, sx = _layer(M, K, N, h, seed=11)
    d_w, d_sw = dev(wq_packed), dev(sw)
    out, ws = pq.pq_linear(dev(x), d_w, d_sw, float(sx), h)
    xq = ws[: M * K // 2].view(M, K // 2).contiguous()
    _, acc = pq.pq_w4a4_gemm(xq, d_w, d_sw, float(sx), want_out=False, want_acc=True)
    acc_ref = O.gemm_i64(O.unpack(host(xq)), O.unpack(wq_packed))
    assert np.array_equal(host(acc).astype(np.int64), acc_ref)
    assert ulp_diff(O.epilogue(acc_ref, np.float32(sx), sw), host(out)).max() <= 1


@pytest.mark.parametrize("name,K,N,h", [("qkv", 4096, 6144, 1), ("o", 4096, 4096, 1), ("gate", 4096, 14336, 1),
                                        ("o_rotated", 4096, 4096, 4096), ("down", 14336, 4096, 128)])
def test_llama3_8b_prefill_8192(pq, name, K, N, h):
    _check_sampled(pq, 8192, K, N, h, seed=12, nsample=16)


# Llama-2-7B at 2048 tokens: q/k/v/o with the full 4096-point rotation online, gate/up to 11008 channels
# (a launch of 40 column panels of 256 and 4 of 192), rotated and as they arrive
@pytest.mark.parametrize("name,K,N,h", [("qkvo", 4096, 4096, 4096), ("gate", 4096, 11008, 4096), ("up", 4096, 11008, 1)])
def test_llama2_7b_prefill_2048(pq, name, K, N, h):
    _check_sampled(pq, 2048, K, N, h, seed=17, nsample=16)


def test_llama2_7b_prefill_2048_down(pq):
    _check_sampled(pq, 2048, 11008, 4096, 128, seed=13, nsample=16)


def test_llama3_70b_prefill_2048_qkv_rotated(pq):
    _check_sampled(pq, 2048, 8192, 10240, 8192, seed=14, nsample=12)


@pytest.mark.parametrize("name,K,N,h", [("o", 8192, 8192, 1), ("gate", 8192, 28672, 1), ("down", 28672, 8192, 128)])
def test_llama3_70b_prefill_2048(pq, name, K, N, h):
    _check_sampled(pq, 2048, K, N, h, seed=18, nsample=8)


@pytest.mark.parametrize("name,K,N,h", [("qkv", 8192, 10240, 1), ("o", 8192, 8192, 1), ("o_rotated", 8192, 8192, 8192),
                                        ("gate", 8192, 28672, 1)])
def test_llama3_70b_decode_one_token(pq, name, K, N, h):
    test_decode_full_shapes(pq, 1, name, K, N, h)


@pytest.mark.parametrize("M", [1, 4, 16])
@pytest.mark.parametrize("name,K,N,h", L3_8B + [("70b_down", 28672, 8192, 128)])
def test_decode_full_shapes(pq, M, name, K, N, h):
    x, wq_packed, sw, sx = _layer(M, K, N, h, seed=21)
    out, ws = pq.pq_linear(dev(x), dev(wq_packed), dev(sw), float(sx), h)
    xq = host(ws)[: M * K // 2].reshape(M, K // 2)
    check_end_to_end(x, wq_packed, sw, sx, h, host(out), xq)
    _, acc = pq.pq_w4a4_gemm(dev(xq), dev(wq_packed), dev(sw), float(sx), want_out=False, want_acc=True)
    assert np.array_equal(host(acc).astype(np.int64), O.gemm_i64(O.unpack(xq), O.unpack(wq_packed)))


# ------------------------------------------------------------------ widened quantizers at the benchmark's sizes
def _sample_rows(M, seed, nsample):
    rng = np.random.default_rng(seed + 1000)
    return np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, size=nsample)]))


@pytest.mark.parametrize("name,K,N,h", [("qkv", 4096, 6144, 1), ("gate", 4096, 14336, 1), ("down", 14336, 4096, 128)])
def test_llama3_8b_prefill_2048_w4a8(pq, name, K, N, h):
    M, seed = 2048, 15
    x = synth.activations(M, K, seed)
    wq, sw = O.weight_rtn(synth.weights(N, K, seed))
    sx = O.calibrate_absmax(synth.calibration(K, seed), h, 8)
    rows = _sample_rows(M, seed, 16)
    out, ws = pq.pq_linear_w4a8(dev(x), dev(O.pack(wq)), dev(sw), float(sx), h)
    codes = host(ws[: M * K].view(M, K)[rows]).view(np.int8)
    out_s = host(out[rows])
    del out, ws
    q_gpu = O.ungroup_even_odd(codes)
    ref = O.linear_bits(x[rows], O.pack(wq), sw, sx, h, 8)
    diff = q_gpu.astype(np.int32) - ref["q"].astype(np.int32)
    idx = np.nonzero(diff)
    assert idx[0].size <= 1e-3 * diff.size and (h > 1 or idx[0].size == 0)
    if idx[0].size:
        t = ref["y"][idx] / np.float64(sx)
        assert np.all(np.abs(diff[idx]) == 1)
        assert np.all(np.abs(t - (np.minimum(q_gpu[idx], ref["q"][idx]) + 0.5)) <= 1e-3)
    o_ref = ref["out"].astype(np.float64)
    assert np.abs(out_s.astype(np.float64) - o_ref).max() <= 1e-2 * np.abs(o_ref).max()
    assert ulp_diff(O.epilogue(O.gemm_i64(q_gpu, wq), sx, sw), out_s).max() <= 1


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("name,K,N,h", [("o", 4096, 4096, 1), ("down", 14336, 4096, 128)])
def test_llama3_8b_prefill_2048_dynamic(pq, bits, name, K, N, h):
    M, seed = 2048, 16
    x = synth.activations(M, K, seed)
    wq, sw = O.weight_rtn(synth.weights(N, K, seed))
    rows = _sample_rows(M, seed, 16)
    out, ws = pq.pq_linear_dynamic(dev(x), dev(O.pack(wq)), dev(sw), h, 1.0, bits)
    total = pq.pq_linear_dynamic_workspace_bytes(M, K, bits)
    s_off = total - ((4 * M + 255) // 256) * 256
    s_gpu = host(ws[s_off: s_off + 4 * M]).view(np.float32)[rows]
    if bits == 8:
        q_gpu = O.ungroup_even_odd(host(ws[: M * K].view(M, K)[rows]).view(np.int8))
    else:
        q_gpu = O.unpack(host(ws[: M * K // 2].view(M, K // 2)[rows]))
    out_s = host(out[rows])
    del out, ws
    ref = O.linear_dynamic(x[rows], O.pack(wq), sw, h, 1.0, bits)
    ia, ib = s_gpu.view(np.int32).astype(np.int64), ref["s"].view(np.int32).astype(np.int64)
    assert np.abs(ia - ib).max() <= (0 if h <= 1 else 4)
    diff = q_gpu.astype(np.int32) - ref["q"].astype(np.int32)
    idx = np.nonzero(diff)
    assert idx[0].size <= 1e-3 * diff.size and (h > 1 or idx[0].size == 0)
    if idx[0].size:
        t = ref["y"][idx] / ref["s"].astype(np.float64)[idx[0]]
        assert np.all(np.abs(diff[idx]) == 1)
        assert np.all(np.abs(t - (np.minimum(q_gpu[idx], ref["q"][idx]) + 0.5)) <= 1e-3)
    o_ref = ref["out"].astype(np.float64)
    assert np.abs(out_s.astype(np.float64) - o_ref).max() <= 1e-2 * np.abs(o_ref).max()
    assert ulp_diff(O.epilogue(O.gemm_i64(q_gpu, wq), s_gpu, sw), out_s).max() <= 1
