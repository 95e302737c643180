#!/usr/bin/env python3
"""Benchmark of the statically quantized W4A4 linear layer on one MI355X.

A step is one pass of the whole path (rotate + quantize + pack, INT4 x INT4 product,
dequantise) over the five linears of one Llama-3-8B block at a 2048-token prefill:
fused qkv 4096->6144, o 4096->4096, gate and up 4096->14336, down 14336->4096.  As in
the paper (App. B) only down_proj rotates online (a block-diagonal 128-point Hadamard,
since 14336 is not a power of two); the other inputs are rotated by matrices absorbed into
the previous layer, so they are quantised as they arrive.  Inputs are seeded synthetic
tensors (paper_2410_05265_amd.synth), resident in HBM before the clock starts.  Before every leg
the GPU is kept busy for 80 ms with a plain matmul (device_warmup): after host-side preparation the
chip needs about 40 ms of load to reach its steady clocks, and the step is 5-15 % slower until then.

The step runs the layer's prepacked path (pq_linear_f6: weights repacked once, offline, into register
images of the 6-bit floating-point matrix instruction, on which the 4-bit codes multiply exactly): per
linear one launch that rotates, quantizes and writes the activations' images, and one product launch.
The two entry points behind pq_linear_f6 are called one after the other so that events can bracket the
product.  The canonical path (pq_linear: nibble-packed weights as they are, INT8 matrix instruction) is
timed beside it.

Prints ONE JSON line: W4A4 linear TOPS for the step (median of REPEATS timed regions of --steps steps),
the roofline of the dominant kernel (the product) from HIP events around its launches inside the timed
regions, an fp16 GEMM of the same shapes on the same GPU, the batch-1 decode bandwidth beside what a
read-only kernel gets on the same bytes, and the CPU oracle timed on a bounded sample.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5033.0      # MI355X dense INT8 MFMA: 256 CU x 2.4 GHz x 8192 ops/clk/CU
FP6_PEAK_TFLOPS = 10066.0    # dense 6-bit (and 4-bit) floating-point MFMA: twice the INT8 rate
HBM_PEAK_GBS = 8000.0
M_PREFILL = 2048
EVENT_EVERY = 25            # steps between two event-instrumented steps of a timed region (each costs ~50 us extra)
REPEATS = 5                 # timed regions of --steps steps each; the median is reported
WEIGHT_SETS = 4             # distinct copies of the block's weights, one per step in turn: with 4 x 163 MB (6-bit
                            # tiles) between two uses of a copy, every step reads its weights from HBM, as the
                            # 32 different blocks of the model do; one copy alone would stay in the 256 MB
                            # memory-side cache
# HBM-side bytes per product launch come from a committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE
# scaled by what the same counters read for a plain copy), not from this run: the file is named in the line.
TRAFFIC_FILE = os.path.join("profiles", "gemm_f6_prefill_llama3_8b_pmc.md")


def traffic_from_profile():
    """The line 'TRAFFIC_BYTES_PER_LAUNCH = <number>' of the committed counter summary, or None."""
    try:
        with open(os.path.join(ROOT, TRAFFIC_FILE)) as f:
            for ln in f:
                if ln.startswith("TRAFFIC_BYTES_PER_LAUNCH"):
                    return float(ln.split("=")[1].split()[0])
    except (OSError, ValueError, IndexError):
        pass
    return None
# name -> (K, N, online Hadamard block)
LINEARS = [("qkv", 4096, 6144, 1), ("o", 4096, 4096, 1), ("gate", 4096, 14336, 1),
           ("up", 4096, 14336, 1), ("down", 14336, 4096, 128)]


# Llama-2-7B block linears (the benchmark configuration's second case): q/k/v (one matrix here) and o behind the
# full 4096-point rotation, gate/up to 11008 channels, down behind 128-point blocks
LINEARS_7B = [("qkv", 4096, 12288, 4096), ("o", 4096, 4096, 4096), ("gate", 4096, 11008, 1),
              ("up", 4096, 11008, 1), ("down", 11008, 4096, 128)]


# Llama-3-70B single-layer linears (the benchmark configuration's large case, one GPU's view of a layer)
LINEARS_70B = [("qkv", 8192, 10240, 1), ("o", 8192, 8192, 1), ("gate", 8192, 28672, 1),
               ("up", 8192, 28672, 1), ("down", 28672, 8192, 128)]


def prepare_layers(torch, synth, M, linears=LINEARS, device_weights=False):
    """Harness-side preparation (offline in a deployment, never timed): RTN per-channel
    4-bit weights with s_w = rowmax/7, and the static step s_x = max|rotated x_cal| / 7
    from a separate 256-token calibration batch.  device_weights: the fp weights are drawn on
    the device (same N(0, 0.02) law, torch's generator) instead of by the seeded host generator,
    which takes minutes for the large matrices; they are quantized the same way."""
    import numpy as np
    layers = []
    for seed, (name, K, N, h) in enumerate(linears):
        x = torch.from_numpy(synth.activations(M, K, seed)).cuda()
        xcal = torch.from_numpy(synth.calibration(K, seed)).cuda().float()
        if device_weights:
            gen = torch.Generator(device="cuda")
            gen.manual_seed(1000 + seed)
            W = torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32) * 0.02
        else:
            W = torch.from_numpy(synth.weights(N, K, seed)).cuda().float()
        if h > 1:
            i = np.arange(h)
            Hm = torch.from_numpy(1.0 - 2.0 * (np.bitwise_count(i[:, None] & i[None, :]) & 1)).float().cuda()
            xcal = (xcal.view(-1, K // h, h) @ Hm).view(-1, K) / (h ** 0.5)
        sx = float(xcal.abs().max().item() / 7.0)
        sw = (W.abs().amax(dim=1) / 7.0).clamp_min(1e-30).float().contiguous()
        q = torch.clamp(torch.round(W / sw[:, None]), -8, 7).to(torch.int32) & 0xF
        wq = (q[:, 0::2] | (q[:, 1::2] << 4)).to(torch.uint8).contiguous()
        layers.append({"name": name, "K": K, "N": N, "h": h, "x": x, "wq": wq, "sw": sw, "sx": sx,
                       "w_f16": W.half().contiguous(),
                       "w6": pq_mod().pq_repack_f6(wq),          # offline: the prepacked weights
                       "x6": torch.empty((pq_mod().pq_f6_tiles_bytes(M, K),), dtype=torch.uint8, device="cuda"),
                       "xq": torch.empty((M, K // 2), dtype=torch.uint8, device="cuda"),
                       "out": torch.empty((M, N), dtype=torch.float16, device="cuda")})
    return layers


def pq_mod():
    import paper_2410_05265_amd.binding as pq
    return pq


DEVICE_WARMUP_MS = 80.0


def device_warmup(torch, ms=DEVICE_WARMUP_MS):
    """Keeps the GPU busy with a plain fp16 matmul for `ms` milliseconds.  After idling (host-side
    preparation) the chip needs ~40 ms of sustained load to reach its steady clocks: measured on the
    headline step, 471 us right after a pause, 441, 425, 417, ... and 400 us from 40 ms on.  Every leg
    and comparator starts from that steady state, so legs are comparable with one another and with the
    driver's own timing of a longer run; the `--warmup` steps of the workload itself come on top."""
    a = getattr(device_warmup, "a", None)
    if a is None:
        a = device_warmup.a = torch.randn((4096, 4096), dtype=torch.float16, device="cuda")
        device_warmup.o = torch.empty_like(a)
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(20):
            torch.matmul(a, a, out=device_warmup.o)
        torch.cuda.synchronize()


def weight_sets(L, key, n):
    """n device copies of a layer's weights (the first is the original)."""
    sets = L.setdefault(key + "_sets", [L[key]])
    while len(sets) < n:
        sets.append(L[key].clone())
    return sets[:n]


def run_prefill(torch, pq, layers, steps, warmup, path="f6", repeats=REPEATS, sets=WEIGHT_SETS):
    """path "f6": pq_rotate_quant_f6 + pq_w4a4_gemm_f6 (the two launches of pq_linear_f6); "int8": pq_rotate_quant +
    pq_w4a4_gemm (those of pq_linear).  Step i multiplies by copy i % sets of the weights.  Returns the median
    seconds per step over `repeats` timed regions, all of them, and the median event-timed duration per linear
    of the product and of the quantizer launch (corrected for the events' own dispatch gap, see below)."""
    wkey = "w6" if path == "f6" else "wq"
    for L in layers:
        weight_sets(L, wkey, sets)
    count = [0]

    def quant(L):
        if path == "f6":
            pq.pq_rotate_quant_f6(L["x"], L["h"], L["sx"], out=L["x6"])
        else:
            pq.pq_rotate_quant(L["x"], L["h"], L["sx"], out=L["xq"])

    def product(L):
        w = L[wkey + "_sets"][count[0] % sets]
        if path == "f6":
            pq.pq_w4a4_gemm_f6(L["x6"], w, L["sw"], L["sx"], L["x"].shape[0], L["N"], L["K"], out=L["out"])
        else:
            pq.pq_w4a4_gemm(L["xq"], w, L["sw"], L["sx"], out=L["out"])

    def step(events=None):
        count[0] += 1
        for L in layers:
            if events is not None:
                q0 = torch.cuda.Event(enable_timing=True)
                q0.record()
            quant(L)
            if events is not None:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            product(L)
            if events is not None:
                e1.record()
                events.append((L["name"], e0, e1))
                events.append(("rq_" + L["name"], q0, e0))

    device_warmup(torch)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    events, regions, gaps = [], [], []
    for _ in range(repeats):
        ev = []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            # an event pair fences the stream (the next launch cannot start under the tail of the
            # previous one), so only every EVENT_EVERY-th step of a timed region carries them
            step(ev if i % EVENT_EVERY == min(EVENT_EVERY, steps) // 2 else None)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        regions.append(dt / steps)
        # what a marker adds to the interval it opens: an instrumented step (first marker to last) against a
        # plain step, spread over its fifteen markers (three per linear; each of the ten timed intervals, quantizer
        # or product, starts at one of them)
        n_inst = len(ev) // (2 * len(layers))
        if n_inst and steps > n_inst:
            first = [e for n, e, _ in ev if n == "rq_" + layers[0]["name"]]
            last = [e for n, _, e in ev if n == layers[-1]["name"]]
            t_inst = sum(a.elapsed_time(b) for a, b in zip(first, last)) * 1e-3 / n_inst
            t_plain = (dt - n_inst * t_inst) / (steps - n_inst)
            gaps.append(max(0.0, (t_inst - t_plain) / (3 * len(layers))))
        events += ev
    per = {}
    for name, e0, e1 in events:
        per.setdefault(name, []).append(e0.elapsed_time(e1) * 1e-3)
    # An event pair around a launch reads the kernel plus the dispatch gap behind the pair's first marker; that gap,
    # measured above in the same timed regions, is taken off every bracketed launch (what remains is what the
    # rocprofv3 kernel trace of the same command shows per launch).
    # (per linear the median over the instrumented launches, not the mean: in the first process on a freshly
    # started machine a few markers are enqueued late by one-time work on the host, which a mean would book as
    # kernel time)
    gap = sorted(gaps)[len(gaps) // 2] if gaps else 0.0
    avg = {k: max(sorted(v)[len(v) // 2] - gap, 1e-9) for k, v in per.items()}
    run_prefill.event_gap = gap
    run_prefill.regions = regions
    return sorted(regions)[len(regions) // 2], {k: v for k, v in avg.items() if not k.startswith("rq_")}, \
        {k[3:]: v for k, v in avg.items() if k.startswith("rq_")}


def run_variants(torch, pq, layers, steps, warmup, ops):
    """The same step through the layer's other entry points: pq_linear_f6 itself (one call per linear), the
    canonical path pq_linear (INT8 matrix instruction), 8-bit static activations (the paper's W4A8 setting),
    per-token dynamic steps (Table 1 row O1) at 4 and 8 bits, gate and up behind one quantizer (pq_linear2_f6), the
    products alone.
    Wall time per step, median of three timed regions; the weights' copies taken in turn as in run_prefill."""
    M = layers[0]["x"].shape[0]
    for L in layers:
        L["xq8"] = torch.empty((M, L["K"]), dtype=torch.int8, device="cuda")
        L["srow"] = torch.empty((M,), dtype=torch.float32, device="cuda")
        L["work"] = torch.empty((max(pq.pq_linear_workspace_bytes(M, L["K"]), pq.pq_linear_f6_workspace_bytes(M, L["K"], L["h"]),
                                     pq.pq_linear_f6_workspace_bytes(M, L["K"], L["K"] if L["h"] <= 1 else L["h"])),),
                                dtype=torch.uint8, device="cuda")

    for L in layers:
        weight_sets(L, "w6", WEIGHT_SETS)
        weight_sets(L, "wq", WEIGHT_SETS)
    count = [0]

    def W(L, key):
        return L[key + "_sets"][count[0] % WEIGHT_SETS]

    def f6_linear():
        for L in layers:
            pq.pq_linear_f6(L["x"], W(L, "w6"), L["sw"], L["sx"], L["h"], out=L["out"], workspace=L["work"])

    def int8_linear():
        for L in layers:
            pq.pq_linear(L["x"], W(L, "wq"), L["sw"], L["sx"], L["h"], out=L["out"], workspace=L["work"])

    def w4a8_static():
        for L in layers:
            pq.pq_rotate_quant8(L["x"], L["h"], L["sx"] * 7.0 / 127.0, out=L["xq8"])
            pq.pq_w4a8_gemm(L["xq8"], W(L, "wq"), L["sw"], L["sx"] * 7.0 / 127.0, out=L["out"])

    def dynamic(bits):
        def step():
            for L in layers:
                q = L["xq8"] if bits == 8 else L["xq"]
                pq.pq_rotate_quant_dynamic(L["x"], L["h"], 1.0, bits, out=q, row_scale=L["srow"])
                pq.pq_gemm_dynamic(q, bits, W(L, "wq"), L["sw"], L["srow"], out=L["out"])
        return step

    # gate and up read the same tensor in the model: pq_linear2_f6 quantizes it once (two products, two outputs)
    gate, up = layers[2], layers[3]

    def gate_up_one_quantizer():
        for L in (layers[0], layers[1]):
            pq.pq_linear_f6(L["x"], W(L, "w6"), L["sw"], L["sx"], L["h"], out=L["out"], workspace=L["work"])
        pq.pq_linear2_f6(gate["x"], W(gate, "w6"), gate["sw"], W(up, "w6"), up["sw"], gate["sx"], gate["h"],
                         out_a=gate["out"], out_b=up["out"], workspace=gate["work"])
        L = layers[4]
        pq.pq_linear_f6(L["x"], W(L, "w6"), L["sw"], L["sx"], L["h"], out=L["out"], workspace=L["work"])

    # the worst case of the benchmark configuration: q/k/v, o, gate and up rotated online as well (their rotation is
    # absorbed into the weights in the paper's pipeline), with the full K-point transform (K = 4096)
    def rotated_everywhere():
        for L in layers:
            h = L["h"] if L["h"] > 1 else L["K"]
            pq.pq_linear_f6(L["x"], W(L, "w6"), L["sw"], L["sx"], h, out=L["out"], workspace=L["work"])

    def f6_products_only():
        for L in layers:
            pq.pq_w4a4_gemm_f6(L["x6"], W(L, "w6"), L["sw"], L["sx"], M, L["N"], L["K"], out=L["out"])

    def int8_products_only():
        for L in layers:
            pq.pq_w4a4_gemm(L["xq"], W(L, "wq"), L["sw"], L["sx"], out=L["out"])

    def counted(fn):
        def step():
            count[0] += 1
            fn()
        return step

    res = {}
    for name, step in (("w4a4_static_f6_linear", f6_linear), ("w4a4_static_int8_linear", int8_linear),
                       ("w4a8_static", w4a8_static), ("w4a4_dynamic", dynamic(4)), ("w4a8_dynamic", dynamic(8)),
                       ("w4a4_static_f6_gate_up_one_quantizer", gate_up_one_quantizer),
                       ("w4a4_static_f6_every_linear_rotated_online", rotated_everywhere),
                       ("w4a4_products_only_f6", f6_products_only), ("w4a4_products_only_int8", int8_products_only)):
        step = counted(step)
        device_warmup(torch)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) / steps)
        dt = sorted(ts)[1]
        res[name] = {"ms_per_step": round(dt * 1e3, 4), "TOPS": round(ops / dt / 1e12, 1)}
    for L in layers:
        del L["xq8"], L["srow"], L["work"]
    return res


def run_prefill_8192(torch, pq, layers, steps=10, warmup=3):
    """The same five linears at M = 8192 tokens (the benchmark configuration's second prefill size): wall time
    per step and per-launch GEMM time from events around every launch."""
    M = 8192
    big = []
    for L in layers:
        x = L["x"].repeat(M // L["x"].shape[0], 1).contiguous()
        big.append(dict(L, x=x, xq=torch.empty((M, L["K"] // 2), dtype=torch.uint8, device="cuda"),
                        x6=torch.empty((pq.pq_f6_tiles_bytes(M, L["K"]),), dtype=torch.uint8, device="cuda"),
                        out=torch.empty((M, L["N"]), dtype=torch.float16, device="cuda")))
    t, g, _ = run_prefill(torch, pq, big, steps, warmup, repeats=3)
    ops = sum(2.0 * M * L["K"] * L["N"] for L in layers)
    return {"ms_per_step": round(t * 1e3, 4), "TOPS": round(ops / t / 1e12, 1),
            "per_linear_TOPS": {L["name"]: round(2.0 * M * L["K"] * L["N"] / g[L["name"]] / 1e12, 1) for L in layers}}


def run_llama2_7b(torch, pq, synth, steps=20, warmup=5):
    """Llama-2-7B block linears at M = 2048 through the whole-layer entry points (the 4096-point rotation of q/k/v/o is
    beyond the tile-writing quantizer's 512, so pq_linear_f6 takes pq_rotate_quant + repack there): wall time per
    step, median of three regions, weights' copies in turn, the fp16 GEMM beside it."""
    layers = prepare_layers(torch, synth, M_PREFILL, LINEARS_7B, device_weights=True)
    ops = sum(2.0 * M_PREFILL * L["K"] * L["N"] for L in layers)
    for L in layers:
        weight_sets(L, "w6", WEIGHT_SETS)
        weight_sets(L, "wq", WEIGHT_SETS)
        L["work"] = torch.empty((max(pq.pq_linear_workspace_bytes(M_PREFILL, L["K"]),
                                     pq.pq_linear_f6_workspace_bytes(M_PREFILL, L["K"], L["h"])),), dtype=torch.uint8, device="cuda")
    count = [0]

    def f6():
        count[0] += 1
        for L in layers:
            pq.pq_linear_f6(L["x"], L["w6_sets"][count[0] % WEIGHT_SETS], L["sw"], L["sx"], L["h"], out=L["out"], workspace=L["work"])

    def int8():
        count[0] += 1
        for L in layers:
            pq.pq_linear(L["x"], L["wq_sets"][count[0] % WEIGHT_SETS], L["sw"], L["sx"], L["h"], out=L["out"], workspace=L["work"])

    res = {"linears": "qkv 4096->12288 and o 4096->4096 (4096-point rotation), gate/up 4096->11008, down 11008->4096 (128-point blocks)"}
    for name, step in (("pq_linear_f6", f6), ("pq_linear", int8)):
        device_warmup(torch)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) / steps)
        dt = sorted(ts)[1]
        res[name] = {"ms_per_step": round(dt * 1e3, 4), "TOPS": round(ops / dt / 1e12, 1)}
    t16 = run_fp16(torch, layers, 5, 2)
    res["fp16_ms_per_step"] = round(t16 * 1e3, 4)
    res["speedup_vs_fp16"] = round(t16 / (res["pq_linear_f6"]["ms_per_step"] * 1e-3), 3)
    return res


def run_llama3_70b(torch, pq, synth, decode=True):
    """The large configuration: Llama-3-70B single-layer linears at M = 2048 prefill (wall time per
    step, per-launch GEMM time from events, the fp16 GEMM beside it) and at batch-1 decode (cold
    weights, HIP graph).  More tiles per launch and more bytes per matrix than the 8B shapes, so
    the fixed cost of a launch weighs less."""
    layers = prepare_layers(torch, synth, M_PREFILL, LINEARS_70B, device_weights=True)
    t, g, _ = run_prefill(torch, pq, layers, 2 * EVENT_EVERY, 3, repeats=3, sets=2)     # 2 x 642 MB of tiles
    ops = sum(2.0 * M_PREFILL * L["K"] * L["N"] for L in layers)
    t16 = run_fp16(torch, layers, 5, 2)
    gemm_ops = sum(2.0 * M_PREFILL * L["K"] * L["N"] for L in layers) / len(layers)
    ach = gemm_ops / (sum(g.values()) / len(g)) / 1e12
    res = {"prefill_2048": {"ms_per_step": round(t * 1e3, 4), "TOPS": round(ops / t / 1e12, 1),
                            "gemm_TOPS_per_launch": round(ach, 1), "gemm_frac_of_int8_peak": round(ach / INT8_PEAK_TOPS, 4),
                            "gemm_frac_of_fp6_peak": round(ach / FP6_PEAK_TFLOPS, 4),
                            "per_linear_us": {L["name"]: round(g[L["name"]] * 1e6, 1) for L in layers},
                            "per_linear_TOPS": {L["name"]: round(2.0 * M_PREFILL * L["K"] * L["N"] / g[L["name"]] / 1e12, 1)
                                                for L in layers},
                            "fp16_ms_per_step": round(t16 * 1e3, 4), "speedup_vs_fp16": round(t16 / t, 3)}}
    if decode:
        for L in layers:
            del L["w_f16"]
        d = run_decode(torch, pq, layers, M=1, floor=True)
        res["decode_M1"] = {"GBps": d["GBps"], "frac_hbm": d["frac_hbm"], "read_only_kernel": d["read_only_kernel"],
                            "per_linear": {k: {"us": v["us"], "frac_hbm": v["frac_hbm"], "read_only_us": v["read_only_us"]}
                                           for k, v in d["per_linear"].items()}}
        # a serving batch: the tiled kernel alone, and with planes for its split-K launch (us per pq_linear)
        a = run_decode(torch, pq, layers, M=64)
        b = run_decode(torch, pq, layers, M=64, planes=True)
        res["serving_M64"] = {"per_linear_us": {k: v["us"] for k, v in a["per_linear"].items()},
                              "per_linear_us_planes": {k: v["us"] for k, v in b["per_linear"].items()},
                              "frac_hbm": a["frac_hbm"], "frac_hbm_planes": b["frac_hbm"]}
    return res


def run_probes(torch, pq):
    """What the GPU delivers on the two bounds with nothing else going on: matrix instructions only
    (INT8 32x32x32, operands of three kinds: the pipe's pace depends on the bits it multiplies), and a
    kernel that only reads 1 GiB from HBM."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    n = 1 << 20
    kinds = {"zeros": torch.zeros(n, dtype=torch.int8, device="cuda"),
             "codes_times_16": (torch.randint(-8, 8, (n,), generator=gen, device="cuda", dtype=torch.int32) * 16).to(torch.int8),
             "random_bytes": torch.randint(-128, 128, (n,), generator=gen, device="cuda", dtype=torch.int32).to(torch.int8)}
    res = {"mfma_only_TOPS": {}}
    for name, t in kinds.items():
        pq.pq_probe_mfma_i8(t, 1000, 256, sink)
        device_warmup(torch)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ops = sum(pq.pq_probe_mfma_i8(t, 1000, 256, sink) for _ in range(5))
        e1.record()
        torch.cuda.synchronize()
        res["mfma_only_TOPS"][name] = round(ops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    # the 6-bit floating-point matrix instruction on the same codes written as E3M2 (exact for -8..8);
    # a register image is 32 bytes: 32 values of 6 bits, little-endian bit stream, in the first 24
    import numpy as np
    rng = np.random.default_rng(7)
    codes = rng.integers(-8, 8, size=(1 << 15, 32))
    table = np.array([0, 12, 16, 18, 20, 21, 22, 23, 24], dtype=np.uint64)        # E3M2 of 0..8
    enc = table[np.abs(codes)] | (np.uint64(32) * (codes < 0).astype(np.uint64))
    words = np.zeros((codes.shape[0], 4), dtype=np.uint64)
    for i in range(32):
        bit = 6 * i
        words[:, bit // 64] |= enc[:, i] << np.uint64(bit % 64)
        if bit % 64 > 58:
            words[:, bit // 64 + 1] |= enc[:, i] >> np.uint64(64 - bit % 64)
    t6 = torch.from_numpy(words.view(np.uint8).reshape(-1)).cuda()
    pq.pq_probe_mfma_f6(t6, 1000, 256, sink)
    device_warmup(torch)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    ops = sum(pq.pq_probe_mfma_f6(t6, 1000, 256, sink) for _ in range(5))
    e1.record()
    torch.cuda.synchronize()
    res["mfma_only_TOPS"]["codes_as_e3m2_6bit_fp32_accumulate"] = round(ops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    big = torch.randint(0, 256, (1 << 30,), generator=gen, device="cuda", dtype=torch.uint8)
    pq.pq_probe_stream_read(big, sink)
    device_warmup(torch, 40.0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    nbytes = sum(pq.pq_probe_stream_read(big, sink) for _ in range(3))
    e1.record()
    torch.cuda.synchronize()
    res["stream_read_GBps"] = round(nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    del big
    return res


def run_fp16(torch, layers, steps, warmup):
    outs = [torch.empty((L["x"].shape[0], L["N"]), dtype=torch.float16, device="cuda") for L in layers]
    device_warmup(torch)

    def step():
        for L, o in zip(layers, outs):
            torch.matmul(L["x"], L["w_f16"].t(), out=o)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def run_int8_ref(torch, layers, steps, warmup):
    """The vendor's plain int8 GEMM on the same five shapes (torch._int_mm -> hipBLASLt): int8 x int8 ->
    int32, nothing to unpack, no dequantising epilogue.  A reference point for what the INT8 matrix pipe
    delivers at these sizes on this GPU."""
    M = layers[0]["x"].shape[0]
    ops_ab = [(torch.randint(-8, 8, (M, L["K"]), dtype=torch.int8, device="cuda"),
               torch.randint(-8, 8, (L["N"], L["K"]), dtype=torch.int8, device="cuda").t()) for L in layers]
    try:
        device_warmup(torch)
        for _ in range(warmup):
            for a, b in ops_ab:
                torch._int_mm(a, b)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            for a, b in ops_ab:
                torch._int_mm(a, b)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps
    except Exception:                                    # comparator only: absent on some builds
        return None


def graph_time(torch, fn, reps=5, inner=20):
    """Microseconds per call of fn, captured `inner` times in a HIP graph (small kernels: the host is not the
    limit); median of `reps` replays."""
    fn()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(inner):
            fn()
    device_warmup(torch, 40.0)
    # then the graph itself for 30 ms: these legs are bound by memory, and after a pause of the memory system (host-side
    # preparation, a compute-bound leg) the first replays run up to 20 % slower than the steady state
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.030:
        graph.replay()
        torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3 / inner)
    return sorted(ts)[len(ts) // 2]


def run_side_rows(torch, pq, synth, T):
    """The rows next to the linear: head-wise rotation of queries, per-head static 4-bit quantization of
    keys (rotated) and values, at Llama-3-8B's attention shape (32 query heads, 8 KV heads, head_dim 128);
    the fused producers (silu(gate) * up -> rotate -> quantize for down_proj, RMS norm -> quantize for a
    4096-channel input); and the on-device MSE grid search for a static step (256 x 14336 calibration
    batch, 50 candidates)."""
    q = torch.from_numpy(synth.activations(T, 4096, 21)).cuda()
    kv = torch.from_numpy(synth.activations(T, 1024, 22)).cuda()
    hs = torch.full((8,), 0.5, dtype=torch.float32, device="cuda")
    qo, ko = torch.empty_like(q), torch.empty((T, 512), dtype=torch.uint8, device="cuda")
    res = {}
    us = graph_time(torch, lambda: pq.pq_rotate_f16(q, 128, out=qo))
    res["q_rotate_f16"] = {"us": round(us, 2), "GBps": round(T * 4096 * 4 / us / 1e3, 1)}
    us = graph_time(torch, lambda: pq.pq_rotate_quant_heads(kv, 8, True, hs, out=ko))
    res["k_rotate_quant_heads"] = {"us": round(us, 2), "GBps": round(T * 1024 * 2.5 / us / 1e3, 1)}
    us = graph_time(torch, lambda: pq.pq_rotate_quant_heads(kv, 8, False, hs, out=ko))
    res["v_quant_heads"] = {"us": round(us, 2), "GBps": round(T * 1024 * 2.5 / us / 1e3, 1)}
    g = torch.from_numpy(synth.activations(T, 14336, 23)).cuda()
    u = torch.from_numpy(synth.activations(T, 14336, 24)).cuda()
    do = torch.empty((T, 7168), dtype=torch.uint8, device="cuda")
    us = graph_time(torch, lambda: pq.pq_silu_mul_rotate_quant(g, u, 128, 0.4, out=do), inner=8)
    res["silu_mul_rotate_quant"] = {"us": round(us, 2), "GBps": round(T * 14336 * 4.5 / us / 1e3, 1)}
    ko2 = torch.empty((T, 2048), dtype=torch.uint8, device="cuda")
    us = graph_time(torch, lambda: pq.pq_rmsnorm_quant(q, 1e-5, 0.4, out=ko2))
    res["rmsnorm_quant"] = {"us": round(us, 2), "GBps": round(T * 4096 * 2.5 / us / 1e3, 1)}
    del g, u, do
    xc = torch.from_numpy(synth.calibration(14336, 4)).cuda()
    t0 = time.perf_counter()
    r = pq.pq_calibrate_static(xc, 128, 4, 50, 0.5)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    r = pq.pq_calibrate_static(xc, 128, 4, 50, 0.5)
    torch.cuda.synchronize()
    res["calibrate_static"] = {"us": round((time.perf_counter() - t1) * 1e6, 1), "tokens": 256, "K": 14336, "n_grid": 50,
                               "gamma_best": round(float(r[2].item()), 3)}
    return res


def replay_median(torch, graph, per, reps=5):
    """Median over `reps` replays of a captured graph, in seconds per captured item (`per` items per replay)."""
    graph.replay()
    torch.cuda.synchronize()
    device_warmup(torch, 40.0)
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e-3 / per)
    return sorted(ts)[len(ts) // 2]


def run_decode(torch, pq, layers, M=1, reps=5, warm=False, planes=False, floor=False):
    """Batch-M decode through pq_linear with cold weights: enough distinct copies of each
    weight matrix that more than 1 GiB is touched before one is reused (the matrices fit
    the 256 MB last-level cache otherwise).  The launches are captured in a HIP graph so
    the host is not the limit; time is per captured launch pair (rotate + streaming GEMM), median of
    `reps` replays.  planes: the workspace also holds the partial-sum planes of the split-K launch.
    floor: the library's read-only kernel (pq_probe_stream_read: 256 workgroups read the bytes once and
    discard them) over the same cold copies, captured and timed the same way: what one launch that only
    streams a matrix of this size costs on this GPU."""
    res = {}
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")

    def measure(L):
        K, N, h = L["K"], L["N"], L["h"]
        nbytes = N * K // 2
        ncopy = max(4, int((1 << 30) // nbytes) + 1)
        # (one allocation for all copies, as a deployment holds its weights in a few large allocations)
        pool = L["wq"].unsqueeze(0).repeat(ncopy, 1, 1)
        ws = [pool[i] for i in range(ncopy)]
        x = L["x"][:M].contiguous()
        out = torch.empty((M, N), dtype=torch.float16, device="cuda")
        wbytes = pq.pq_linear_workspace_bytes_split(M, N, K) if planes else pq.pq_linear_workspace_bytes(M, K)
        work = torch.empty((max(256, wbytes),), dtype=torch.uint8, device="cuda")
        pq.pq_linear(x, ws[0], L["sw"], L["sx"], h, out=out, workspace=work)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for w in ws:
                pq.pq_linear(x, w, L["sw"], L["sx"], h, out=out, workspace=work)
        t = replay_median(torch, graph, ncopy, reps)
        res[L["name"]] = {"us": round(t * 1e6, 2), "GBps": round(nbytes / t / 1e9, 1),
                          "frac_hbm": round(nbytes / t / 1e9 / HBM_PEAK_GBS, 3)}
        del graph
        if floor:
            pq.pq_probe_stream_read(ws[0].view(-1), sink)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for w in ws:
                    pq.pq_probe_stream_read(w.view(-1), sink)
            tf = replay_median(torch, graph, ncopy, reps)
            res[L["name"]].update({"read_only_us": round(tf * 1e6, 2), "read_only_GBps": round(nbytes / tf / 1e9, 1),
                                   "over_read_only": round(t / tf, 3)})
            del graph
        if warm:
            # one weight buffer replayed: it stays in the last-level cache ("warm / LLC", not an HBM figure)
            w0 = ws[0]
            us = graph_time(torch, lambda: pq.pq_linear(x, w0, L["sw"], L["sx"], h, out=out, workspace=work), inner=32)
            res[L["name"]]["warm_llc_us"] = round(us, 2)
        del ws, pool

    # The first graph-timed sequence of fused launches in a process reads up to 20 % slower than the same
    # sequence measured again (same library, same buffers, after any amount of warm-up; the read-only kernel
    # timed right behind it is not affected): the leg's first linear is therefore measured once untimed.
    if not getattr(run_decode, "primed", False):
        run_decode.primed = True
        measure(layers[0])
        res.clear()
    for L in layers:
        measure(L)
    tot_b = sum(L["N"] * L["K"] // 2 for L in layers)
    tot_t = sum(v["us"] for v in res.values()) * 1e-6
    r = {"M": M, "weights": "cold (>1 GiB cycled)", "timing": "median of %d graph replays" % reps, "per_linear": res,
         "GBps": round(tot_b / tot_t / 1e9, 1), "frac_hbm": round(tot_b / tot_t / 1e9 / HBM_PEAK_GBS, 3)}
    if floor:
        tf = sum(v["read_only_us"] for v in res.values()) * 1e-6
        r["read_only_kernel"] = {"GBps": round(tot_b / tf / 1e9, 1), "frac_hbm": round(tot_b / tf / 1e9 / HBM_PEAK_GBS, 3),
                                 "note": "256 workgroups read the same cold bytes once and discard them: one launch's floor"}
    return r


def run_decode_pair(torch, pq, a, b, M=1, reps=5):
    """gate and up through pq_linear2: one launch streams both matrices (separate buffers, separate outputs).
    Cold copies, HIP graph and timing as in run_decode; the floor is the read-only kernel over both copies."""
    K, h = a["K"], a["h"]
    nbytes = (a["N"] + b["N"]) * K // 2
    ncopy = max(4, int((1 << 30) // nbytes) + 1)
    pool_a, pool_b = a["wq"].unsqueeze(0).repeat(ncopy, 1, 1), b["wq"].unsqueeze(0).repeat(ncopy, 1, 1)
    wa, wb = [pool_a[i] for i in range(ncopy)], [pool_b[i] for i in range(ncopy)]
    x = a["x"][:M].contiguous()
    oa = torch.empty((M, a["N"]), dtype=torch.float16, device="cuda")
    ob = torch.empty((M, b["N"]), dtype=torch.float16, device="cuda")
    work = torch.empty((max(256, pq.pq_linear_workspace_bytes(M, K)),), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")

    def call(i):
        pq.pq_linear2(x, wa[i], a["sw"], wb[i], b["sw"], a["sx"], h, out_a=oa, out_b=ob, workspace=work)

    call(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(ncopy):
            call(i)
    t = replay_median(torch, graph, ncopy, reps)
    del graph
    pq.pq_probe_stream_read(wa[0].view(-1), sink)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(ncopy):
            pq.pq_probe_stream_read(wa[i].view(-1), sink)
            pq.pq_probe_stream_read(wb[i].view(-1), sink)
    tf = replay_median(torch, graph, ncopy, reps)
    return {"us": round(t * 1e6, 2), "GBps": round(nbytes / t / 1e9, 1), "frac_hbm": round(nbytes / t / 1e9 / HBM_PEAK_GBS, 3),
            "read_only_two_launches_us": round(tf * 1e6, 2), "entry_point": "pq_linear2"}


def cpu_baseline(synth, rows=256):
    """The CPU oracle as it stands, on the first `rows` tokens of the same five linears."""
    import numpy as np
    import oracle as O
    prepared = []
    for seed, (name, K, N, h) in enumerate(LINEARS):
        x = synth.activations(rows, K, seed)
        rng = np.random.default_rng([seed, 9])
        wq_packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
        prepared.append((x, wq_packed, synth.random_scales(N, seed), np.float32(0.3), h))
    stage = {"rotate": 0.0, "quantize+pack": 0.0, "product": 0.0, "epilogue": 0.0}
    t0 = time.perf_counter()
    for x, wq_packed, sw, sx, h in prepared:          # O.linear, stage by stage
        a = time.perf_counter()
        y = O.rotate(x, h)
        b = time.perf_counter()
        q = O.quantize(y, sx)
        O.pack(q)
        c = time.perf_counter()
        acc = O.gemm_i64(q, O.unpack(wq_packed))
        d = time.perf_counter()
        O.epilogue(acc, np.float32(sx), sw)
        e = time.perf_counter()
        for k, v in zip(stage, (b - a, c - b, d - c, e - d)):
            stage[k] += v
    dt = time.perf_counter() - t0
    ops = sum(2.0 * rows * K * N for _, K, N, _ in LINEARS)
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
    except OSError:
        pass
    return {"value": round(ops / dt / 1e12, 5), "unit": "TOPS", "cores": O.threads(), "cpu_model": model,
            "kind": "oracle",
            "sample": "first %d of 2048 tokens, all five linears, whole path (fp64 dense Hadamard, RNE, int64 "
                      "product, fp64 epilogue), %.1f s: %s" % (rows, dt, ", ".join("%s %.1f s" % kv for kv in stage.items()))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-variants", action="store_true", help="skip the W4A8 / per-token dynamic variants of the step")
    ap.add_argument("--serving-only", action="store_true",
                    help="of the side legs run only serving_batch (32..256 tokens); for profiles")
    ap.add_argument("--cpu-rows", type=int, default=2048, help="tokens of the workload the CPU oracle is timed on (all 2048: about 12 s)")
    ap.add_argument("--headline-only", action="store_true",
                    help="run the headline leg alone (no comparators, no side legs): for profiles, where every "
                         "k_gemm_f6 launch then belongs to the headline step, in the order qkv, o, gate, up, down")
    ap.add_argument("--profile-copy", action="store_true",
                    help="also run a plain 256 MiB elementwise copy (calibrates HBM counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path shards over tokens or channels without "
              "changing the kernel); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_05265_amd import synth
    import paper_2410_05265_amd.binding as pq
    pq.lib()                                   # fails loudly if libpq.so is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    if args.profile_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    layers = prepare_layers(torch, synth, M_PREFILL)
    ops = sum(2.0 * M_PREFILL * L["K"] * L["N"] for L in layers)
    t_step, gemm_t, rq_t = run_prefill(torch, pq, layers, args.steps, args.warmup)
    event_gap = run_prefill.event_gap
    t_fp16 = None if args.headline_only else run_fp16(torch, layers, max(5, args.steps // 2), max(2, args.warmup // 2))

    gemm_ops = {L["name"]: 2.0 * M_PREFILL * L["K"] * L["N"] for L in layers}
    avg_ops = sum(gemm_ops.values()) / len(gemm_ops)
    avg_dur = sum(gemm_t.values()) / len(gemm_t)
    achieved = avg_ops / avg_dur / 1e12                              # durations: events minus their dispatch gap
    achieved_raw = avg_ops / (avg_dur + event_gap) / 1e12
    traffic = traffic_from_profile()
    result = {
        "metric": "W4A4 linear TOPS + speedup vs fp16 GEMM, Llama-3-8B 2048-tok prefill; decode GB/s",
        "value": round(ops / t_step / 1e12, 1), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(t_step * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 codes as E3M2 on the 6-bit floating-point MFMA, fp32 accumulate (exact: integer sums below 2^24)",
        "data": "synthetic",
        "timing": {"repeats": REPEATS, "ms_per_step_all": [round(t * 1e3, 4) for t in run_prefill.regions],
                   "note": "%d timed regions of --steps steps each, synchronised on both sides; ms_per_step and value are the median region"
                           % REPEATS},
        "device_warmup_ms": DEVICE_WARMUP_MS,
        "config": {"workload": "Llama-3-8B block linears, M=2048 prefill: qkv 4096->6144, o 4096->4096, "
                               "gate/up 4096->14336, down 14336->4096 (online 128-point block Hadamard on down only)",
                   "tokens": M_PREFILL,
                   "weights": "%d copies of the block's weights, one per step in turn: every step reads its weights from HBM" % WEIGHT_SETS,
                   "path": "pq_linear_f6 (weights prepacked offline as f6 tiles): per linear "
                                                "pq_rotate_quant_f6 + pq_w4a4_gemm_f6"},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 1), "peak": FP6_PEAK_TFLOPS, "unit": "TOPS",
                     "frac": round(achieved / FP6_PEAK_TFLOPS, 4),
                     "peak_note": "the contraction runs on the 6-bit floating-point matrix instruction: its own dense peak",
                     "int8_peak": INT8_PEAK_TOPS, "frac_of_int8_peak": round(achieved / INT8_PEAK_TOPS, 4),
                     "traffic": traffic, "traffic_source": TRAFFIC_FILE if traffic is not None else None,
                     "kernel": "k_gemm_f6 (five launches per step, averaged per launch; HIP events around the "
                               "launches of every %dth step of the timed regions, minus the dispatch gap an event "
                               "pair adds, measured in the same regions)" % EVENT_EVERY,
                     "avg_launch_us": round(avg_dur * 1e6, 2),
                     "event_gap_us": round(event_gap * 1e6, 2),
                     "achieved_events_uncorrected": round(achieved_raw, 1),
                     "per_linear_TOPS": {k: round(gemm_ops[k] / v / 1e12, 1) for k, v in gemm_t.items()},
                     "per_linear_frac_of_int8_peak": {k: round(gemm_ops[k] / v / 1e12 / INT8_PEAK_TOPS, 4) for k, v in gemm_t.items()},
                     "per_linear_us": {k: round(v * 1e6, 1) for k, v in gemm_t.items()}},
        "rotate_quant": {"bound": "hbm", "kernel": "k_rotate_quant_f6", "per_linear_us": {k: round(v * 1e6, 1) for k, v in rq_t.items()},
                         "per_linear_GBps": {L["name"]: round(M_PREFILL * L["K"] * 2.75 / rq_t[L["name"]] / 1e9, 1)
                                             for L in layers},
                         "note": "pq_rotate_quant_f6 launches of the instrumented steps; 2.75 algorithmic bytes per element "
                                 "(2 read, 0.75 written as 6-bit images)"},
        "fp16_gemm": None if t_fp16 is None else {"ms_per_step": round(t_fp16 * 1e3, 4), "TFLOPS": round(ops / t_fp16 / 1e12, 1),
                      "frac_of_fp16_peak": round(ops / t_fp16 / 1e12 / (INT8_PEAK_TOPS / 2), 4),
                      "speedup_pq_linear": round(t_fp16 / t_step, 3),
                      "speedup_pq_w4a4_gemm_only": round(t_fp16 / sum(gemm_t.values()), 3), "impl": "torch.matmul fp16"},
    }

    def canonical_leg():
        # the canonical path: nibble-packed weights as they are, product on the INT8 matrix instruction
        t8, g8, r8 = run_prefill(torch, pq, layers, args.steps, max(2, args.warmup // 2), path="int8", repeats=3)
        a8 = avg_ops / (sum(g8.values()) / len(g8)) / 1e12
        return {"path": "pq_linear: per linear pq_rotate_quant + pq_w4a4_gemm (k_gemm_dma / k_gemm_dual)",
                "ms_per_step": round(t8 * 1e3, 4), "TOPS": round(ops / t8 / 1e12, 1),
                "product_TOPS_per_launch": round(a8, 1), "product_frac_of_int8_peak": round(a8 / INT8_PEAK_TOPS, 4),
                "per_linear_us": {k: round(v * 1e6, 1) for k, v in g8.items()},
                "rotate_quant_us": {k: round(v * 1e6, 1) for k, v in r8.items()},
                "headline_over_this": round(t8 / t_step, 3)}

    def one_copy_leg():
        t1, g1, _ = run_prefill(torch, pq, layers, args.steps, max(2, args.warmup // 2), repeats=3, sets=1)
        a1 = avg_ops / (sum(g1.values()) / len(g1)) / 1e12
        return {"note": "the same step with ONE copy of the weights used every step: its 163 MB of tiles then stay in the "
                        "256 MB memory-side cache between steps, which a model of 32 different blocks does not offer; "
                        "context, not the headline",
                "ms_per_step": round(t1 * 1e3, 4), "TOPS": round(ops / t1 / 1e12, 1),
                "product_TOPS_per_launch": round(a1, 1), "product_frac_of_int8_peak": round(a1 / INT8_PEAK_TOPS, 4),
                "per_linear_us": {k: round(v * 1e6, 1) for k, v in g1.items()}}

    # Everything below is a side leg: a failure there is recorded in its place and never costs the line.
    def leg(key, fn):
        try:
            result[key] = fn()
        except Exception as e:                           # noqa: BLE001 (reported, not swallowed)
            result[key] = {"error": "%s: %s" % (type(e).__name__, e)}
            print("bench.py: leg %s failed: %r" % (key, e), file=sys.stderr)
        return result[key]

    def int8_leg():
        t_i8 = run_int8_ref(torch, layers, max(5, args.steps // 2), max(2, args.warmup // 2))
        if t_i8 is None:
            return {"error": "torch._int_mm not available"}
        return {"ms_per_step": round(t_i8 * 1e3, 4), "TOPS": round(ops / t_i8 / 1e12, 1),
                "pq_gemm_only_ms": round(sum(gemm_t.values()) * 1e3, 4),
                "impl": "torch._int_mm (hipBLASLt): int8 x int8 -> int32, no unpack, no epilogue"}

    def probes_leg():
        pr = run_probes(torch, pq)
        pr["product_kernel_frac_of_mfma_only_e3m2"] = round(achieved / pr["mfma_only_TOPS"]["codes_as_e3m2_6bit_fp32_accumulate"], 4)
        return pr

    def variants_leg():
        v = run_variants(torch, pq, layers, max(5, args.steps // 2), max(2, args.warmup // 2), ops)
        v["dynamic_over_static_w4a4"] = round(v["w4a4_dynamic"]["ms_per_step"] / result["ms_per_step"], 3)
        return v

    def decode_leg():
        dec = run_decode(torch, pq, layers, M=1, warm=True, floor=True)
        # gate and up share their input: pq_linear2 streams both matrices in one launch
        gu = run_decode_pair(torch, pq, layers[2], layers[3], M=1)
        pl = dec["per_linear"]
        t_block = (pl["qkv"]["us"] + pl["o"]["us"] + gu["us"] + pl["down"]["us"]) * 1e-6
        b_block = sum(L["N"] * L["K"] // 2 for L in layers)
        dec["gate_up_one_launch"] = dict(gu, block_GBps=round(b_block / t_block / 1e9, 1),
                                         block_frac_hbm=round(b_block / t_block / 1e9 / HBM_PEAK_GBS, 3))
        if "stream_read_GBps" in result.get("achievable", {}):
            result["achievable"]["decode_frac_of_stream_read"] = round(dec["GBps"] / result["achievable"]["stream_read_GBps"], 4)
            # the read-only kernel on one cold matrix of each size: what a single launch that streams that many bytes costs
            result["achievable"]["stream_read_at_size"] = {
                "%.1f MB" % (L["N"] * L["K"] / 2 / 1e6): {"us": pl[L["name"]]["read_only_us"], "GBps": pl[L["name"]]["read_only_GBps"]}
                for L in layers}
        for m in (4, 16):
            d = run_decode(torch, pq, layers, M=m)
            dec["M%d" % m] = {"GBps": d["GBps"], "frac_hbm": d["frac_hbm"],
                              "per_linear_us": {k: v["us"] for k, v in d["per_linear"].items()}}
        return dec

    def serving_leg():
        # between decode and prefill: the tiled kernel alone, and with planes for its split-K launch
        res = {"note": "pq_linear, cold weights, us per linear; 'planes': workspace of pq_linear_workspace_bytes_split"}
        for m in (32, 64, 128, 256):
            a = run_decode(torch, pq, layers, M=m)
            b = run_decode(torch, pq, layers, M=m, planes=True)
            res["M%d" % m] = {"per_linear_us": {k: v["us"] for k, v in a["per_linear"].items()},
                              "per_linear_us_planes": {k: v["us"] for k, v in b["per_linear"].items()},
                              "frac_hbm": a["frac_hbm"], "frac_hbm_planes": b["frac_hbm"]}
        return res

    if args.headline_only:
        print(json.dumps(result))
        return
    if args.serving_only:
        args.no_variants = args.no_cpu = True
    else:
        leg("int8_gemm", int8_leg)
    if not args.serving_only:
        leg("canonical_int8_path", canonical_leg)
        leg("weights_cache_resident", one_copy_leg)
    if not args.no_variants:
        leg("achievable", probes_leg)
        leg("prefill_8192", lambda: run_prefill_8192(torch, pq, layers))
        leg("side_rows", lambda: run_side_rows(torch, pq, synth, M_PREFILL))
        leg("variants", variants_leg)
    if not args.no_decode and not args.serving_only:
        leg("decode", decode_leg)
    if args.serving_only or not (args.no_decode or args.no_variants):
        leg("serving_batch", serving_leg)
    if not args.no_variants:
        del layers
        torch.cuda.empty_cache()
        leg("llama2_7b", lambda: run_llama2_7b(torch, pq, synth))
        torch.cuda.empty_cache()
        leg("llama3_70b", lambda: run_llama3_70b(torch, pq, synth, decode=not args.no_decode))
    if not args.no_cpu:
        leg("cpu_baseline", lambda: cpu_baseline(synth, args.cpu_rows))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
