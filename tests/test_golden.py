"""The fixtures under tests/golden/.

worked_examples.txt: values computed by hand from the paper's definitions (App. B rotation, Eq. 1
quantizer, nibble layout, integer product, Table 1 row O2 epilogue).  The oracle must reproduce them
(CPU), and so must the HIP path (GPU).
tiny_16x512x512.txt: what the oracle computed for the smallest benchmark configuration, written by
tests/golden/make_tiny.py; pins the oracle against accidental changes (CPU) and is a second route
by which the HIP path is compared with it (GPU: accumulators of the stored codes exactly, the
layer's own codes equal to the stored ones up to rounding ties).
"""

import os

import numpy as np
import pytest

import oracle as O

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_records(name):
    rec = {}
    with open(os.path.join(HERE, name)) as f:
        for line in f:
            if line.startswith("#") or ":" not in line:
                continue
            k, v = line.split(":", 1)
            rec[k.strip()] = v.strip()
    return rec


def nums(s, dtype=np.float64):
    return np.array([[float(t) for t in row.split()] for row in s.split("/")], dtype=dtype)


W = read_records("worked_examples.txt")


def test_oracle_reproduces_the_worked_examples():
    assert np.array_equal(O.rotate(nums(W["hadamard4_x"], np.float16), 4), nums(W["hadamard4_y"]))
    assert np.array_equal(O.rotate(nums(W["hadamard4x2_x"], np.float16), 4), nums(W["hadamard4x2_y"]))
    s = np.float32(W["quant_s"])
    assert np.array_equal(O.quantize(nums(W["quant_x"], np.float16), s), nums(W["quant_q"], np.int8))
    packed = O.pack(nums(W["pack_q"], np.int8))
    assert packed.tobytes().hex() == W["pack_bytes_hex"].replace(" ", "")
    assert np.array_equal(O.unpack(packed), nums(W["pack_q"], np.int8))
    acc = O.gemm_i64(nums(W["gemm_x"], np.int8), nums(W["gemm_w"], np.int8))
    assert np.array_equal(acc, nums(W["gemm_acc"], np.int64))
    out = O.epilogue(acc, np.float32(W["epi_sx"]), nums(W["epi_sw"], np.float32)[0])
    assert np.array_equal(out.astype(np.float64), nums(W["epi_out"]))


def test_oracle_still_computes_the_stored_tiny_configuration():
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_tiny", os.path.join(HERE, "make_tiny.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = read_records("tiny_16x512x512.txt")
    for k, v in mod.records():
        assert stored[k] == v, k


@pytest.mark.gpu
def test_hip_path_reproduces_the_worked_examples():
    import paper_2410_05265_amd.binding as pq
    from pq_testlib import dev, host
    pq.lib()
    # rotation + quantizer: a row of 32 channels (the call's minimum) made of the worked blocks;
    # with step 1/2^k the rotated integers and halves quantize exactly
    x = np.tile(nums(W["hadamard4x2_x"], np.float16), (1, 4))
    want = np.tile(nums(W["hadamard4x2_y"]), (1, 4))
    codes = O.unpack(host(pq.pq_rotate_quant(dev(x), 4, 1.0)))
    assert np.array_equal(codes, np.clip(np.rint(want), -8, 7).astype(np.int8))
    xq = np.zeros((1, 32), np.float16)
    xq[0, :12] = nums(W["quant_x"], np.float16)[0]
    codes = O.unpack(host(pq.pq_rotate_quant(dev(xq), 1, float(W["quant_s"]))))
    assert np.array_equal(codes[0, :12], nums(W["quant_q"], np.int8)[0]) and not codes[0, 12:].any()
    # product + epilogue: the worked 2 x 4 by 3 x 4 example padded with zero codes to K = 32, N = 16
    xc = np.zeros((2, 32), np.int8); xc[:, :4] = nums(W["gemm_x"], np.int8)
    wc = np.zeros((16, 32), np.int8); wc[:3, :4] = nums(W["gemm_w"], np.int8)
    sw = np.ones(16, np.float32); sw[:3] = nums(W["epi_sw"], np.float32)[0]
    for variant in (0, 2, 3):
        prev = pq.pq_set_gemm_variant(variant)
        try:
            out, acc = pq.pq_w4a4_gemm(dev(O.pack(xc)), dev(O.pack(wc)), dev(sw), float(W["epi_sx"]), want_out=True,
                                       want_acc=True)
        finally:
            pq.pq_set_gemm_variant(prev)
        assert np.array_equal(host(acc)[:, :3], nums(W["gemm_acc"], np.int32)) and not host(acc)[:, 3:].any()
        assert np.array_equal(host(out)[:, :3].astype(np.float64), nums(W["epi_out"]))


@pytest.mark.gpu
def test_hip_path_against_the_stored_tiny_configuration():
    import hashlib
    import paper_2410_05265_amd.binding as pq
    from paper_2410_05265_amd import synth
    from pq_testlib import dev, host
    pq.lib()
    stored = read_records("tiny_16x512x512.txt")
    M, K, N, H = 16, 512, 512, 512
    x = synth.activations(M, K, 0)
    wq, sw = O.weight_rtn(synth.weights(N, K, 0))
    sx = np.frombuffer(bytes.fromhex(stored["act_scale_f32_hex"]), np.float32)[0]
    out, work = pq.pq_linear(dev(x), dev(O.pack(wq)), dev(sw), float(sx), H)
    codes = O.unpack(host(work)[:M * K // 2].reshape(M, K // 2))
    want_row0 = np.array(stored["codes_row0_first16"].split(), np.int64)
    sha = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
    if sha(O.pack(codes)) == stored["codes_packed_sha256"]:
        # same codes as the oracle's: then accumulators and outputs are fixed too
        _, acc = pq.pq_w4a4_gemm(dev(O.pack(codes)), dev(O.pack(wq)), dev(sw), float(sx), want_out=False, want_acc=True)
        assert sha(host(acc)) == stored["acc_int32_sha256"]
        assert " ".join(np.float16(v).tobytes().hex() for v in host(out)[0, :8]) == stored["out_row0_first8_f16_hex"]
        assert sha(host(out)) == stored["out_f16_sha256"]
    else:
        # a rotated value on a rounding tie may fall to the other side in fp32: then the differing codes are few,
        # off by one, and each within 1e-3 of a half-integer of the oracle's fp64 quotient; the outputs follow from
        # the GPU's own codes through the oracle's product and epilogue (pq_testlib.check_end_to_end)
        from pq_testlib import check_end_to_end
        nflip, _ = check_end_to_end(x, O.pack(wq), sw, sx, H, host(out), O.pack(codes))
        assert 0 < nflip <= 1e-3 * M * K and np.abs(codes[0, :16] - want_row0).max() <= 1
