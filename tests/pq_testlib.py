"""Helpers shared by the GPU parity tests (inputs from synth, expectations from the oracle)."""

import numpy as np
import torch

import oracle as O
from paper_2410_05265_amd import synth


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def f16_ordinal(a):
    """Map fp16 values to integers that are consecutive for consecutive floats."""
    b = np.asarray(a, dtype=np.float16).view(np.uint16).astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def ulp_diff(a, b):
    return np.abs(f16_ordinal(a) - f16_ordinal(b))


def prepare_layer(M, K, N, h, seed=0):
    """Seeded layer: fp16 activations, calibrated static step, packed RTN weights (oracle, CPU)."""
    x = synth.activations(M, K, seed)
    xcal = synth.calibration(K, seed)
    W = synth.weights(N, K, seed)
    wq, sw = O.weight_rtn(W)
    sx = O.calibrate_absmax(xcal, h)
    return {"x": x, "wq": wq, "wq_packed": O.pack(wq), "sw": sw, "sx": sx, "h": h}


def check_end_to_end(x, wq_packed, sw, sx, h, out_gpu, xq_gpu, tau=1e-3, max_flip_frac=1e-3):
    """Gate B: code flips only at rounding ties, output close, and the GPU's own codes
    reproduce the GPU's output through the oracle's product and epilogue."""
    ref = O.linear(x, wq_packed, sw, sx, h, return_all=True)
    q_gpu = O.unpack(xq_gpu)
    diff = q_gpu.astype(np.int32) - ref["q"].astype(np.int32)
    flips = np.nonzero(diff)
    nflip = flips[0].size
    assert nflip <= max_flip_frac * diff.size, "too many differing codes: %d of %d" % (nflip, diff.size)
    if nflip:
        assert np.all(np.abs(diff[flips]) == 1)
        t = ref["y"][flips] / np.float64(sx)
        lo = np.minimum(q_gpu[flips], ref["q"][flips]).astype(np.float64)
        assert np.all(np.abs(t - (lo + 0.5)) <= tau), "a code differs away from a rounding tie"
    o_ref = ref["out"].astype(np.float64)
    o_gpu = out_gpu.astype(np.float64)
    rel = np.max(np.abs(o_gpu - o_ref)) / max(np.max(np.abs(o_ref)), 1e-30)
    assert rel <= 1e-2, "max error relative to max|out| is %g" % rel
    # code substitution: the oracle's product + epilogue on the GPU's codes gives the GPU's output
    sub = O.epilogue(O.gemm_i64(q_gpu, O.unpack(wq_packed)), np.float32(sx), sw)
    assert ulp_diff(sub, out_gpu).max() <= 1
    return nflip, rel
