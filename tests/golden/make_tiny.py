"""Writes tests/golden/tiny_16x512x512.txt: what the CPU oracle computes for the smallest benchmark
configuration (16 tokens, 512 -> 512 channels, full 512-point rotation, seeded synthetic inputs).
Calls only `oracle/` and the seeded input generators.  The stored values pin the oracle against
later accidental changes of its arithmetic; the GPU tests compare the HIP path with the same file.

    python tests/golden/make_tiny.py
"""

import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle as O                                   # noqa: E402
from paper_2410_05265_amd import synth               # noqa: E402

M, K, N, H, SEED = 16, 512, 512, 512, 0


def compute():
    x = synth.activations(M, K, SEED)
    wq, sw = O.weight_rtn(synth.weights(N, K, SEED))
    sx = O.calibrate_absmax(synth.calibration(K, SEED), H)
    ref = O.linear(x, O.pack(wq), sw, sx, H, return_all=True)
    return x, wq, sw, sx, ref


def records():
    x, wq, sw, sx, ref = compute()
    q, acc, out = ref["q"], O.gemm_i64(ref["q"], wq), ref["out"]
    sha = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
    return [
        ("config", "M=%d K=%d N=%d had_block=%d seed=%d" % (M, K, N, H, SEED)),
        ("act_scale_f32_hex", np.float32(sx).tobytes().hex()),
        ("codes_row0_first16", " ".join(str(int(v)) for v in q[0, :16])),
        ("codes_histogram_-8..7", " ".join(str(int((q == v).sum())) for v in range(-8, 8))),
        ("codes_packed_sha256", sha(O.pack(q))),
        ("acc_row0_first8", " ".join(str(int(v)) for v in acc[0, :8])),
        ("acc_int32_sha256", sha(acc.astype(np.int32))),
        ("out_row0_first8_f16_hex", " ".join(np.float16(v).tobytes().hex() for v in out[0, :8])),
        ("out_f16_sha256", sha(out.astype(np.float16))),
    ]


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_16x512x512.txt")
    with open(path, "w") as f:
        f.write("# written by tests/golden/make_tiny.py from the CPU oracle alone; do not edit\n")
        for k, v in records():
            f.write("%s: %s\n" % (k, v))
    print(open(path).read())
