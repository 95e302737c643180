"""The C ABI: every symbol include/pq.h declares is exported, host-only calls work without
a GPU, and argument errors come back as status codes with nothing launched."""

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def b():
    import paper_2410_05265_amd.binding as binding
    from paper_2410_05265_amd import build
    if build.is_stale():
        build.build_lib()
    binding.lib()
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pq_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_exported_and_bound(b):
    names = declared_symbols()
    assert {"pq_rotate_quant", "pq_w4a4_gemm", "pq_linear"} <= set(names)
    raw = ctypes.CDLL(b.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
        assert n in b.SIGNATURES, n
        assert hasattr(b, n) or n in ("pq_version", "pq_status_str"), n


def test_host_only_calls(b):
    L = b.lib()
    assert L.pq_version() >= 100
    assert b.status_str(0) == "PQ_OK" and b.status_str(4) == "PQ_ERR_SCALE" and b.status_str(99) == "PQ_ERR_UNKNOWN"
    assert L.pq_linear_workspace_bytes(0, 4096) == 0
    assert L.pq_linear_workspace_bytes(1, 512) == 256
    assert L.pq_linear_workspace_bytes(3, 4096) == 6144
    assert L.pq_linear_workspace_bytes(2048, 14336) == 2048 * 7168
    assert L.pq_set_gemm_variant(9) == -1 and L.pq_set_gemm_variant(0) == 0
    # planes of partial sums for the split launch: none for decode and prefill, some in between
    wsb = L.pq_w4a4_gemm_workspace_bytes
    assert wsb(1, 4096, 4096) == 0 and wsb(16, 4096, 14336) == 0 and wsb(2048, 4096, 14336) == 0
    for m in (24, 64):       # a whole number of [m, 4096] int32 planes, how many is the cost model's business
        assert wsb(m, 4096, 14336) % (m * 4096 * 4) == 0 and 2 <= wsb(m, 4096, 14336) // (m * 4096 * 4) <= 32
    assert wsb(64, 4096, 14336 + 32) == 0 and wsb(64, 4090, 4096) == 0 and wsb(-1, 4096, 4096) == 0
    assert L.pq_linear_workspace_bytes_split(64, 4096, 14336) == 64 * 7168 + wsb(64, 4096, 14336)
    assert L.pq_linear_workspace_bytes_split(2048, 4096, 14336) == 2048 * 7168
    gwb = L.pq_gemm_workspace_bytes
    assert gwb(64, 4096, 14336, 4) == wsb(64, 4096, 14336) and gwb(64, 4096, 14336, 8) % (64 * 4096 * 4) == 0
    assert gwb(64, 4096, 14336, 8) > 0 and gwb(64, 4096, 14336, 6) == 0 and gwb(2048, 4096, 14336, 8) == 0
    assert L.pq_linear_w4a8_workspace_bytes_split(64, 4096, 14336) == 64 * 14336 + gwb(64, 4096, 14336, 8)
    assert L.pq_linear_dynamic_workspace_bytes_split(64, 4096, 14336, 4) == 64 * 7168 + 256 + gwb(64, 4096, 14336, 4)
    assert L.pq_linear_dynamic_workspace_bytes_split(64, 4096, 14336, 5) == 0
    assert L.pq_set_gemm_variant(5) == 0
    assert wsb(100, 256, 2048) == 5 * 100 * 256 * 4 and wsb(100, 256, 384) == 0
    assert L.pq_set_gemm_variant(0) == 5
    assert L.pq_linear_w4a8_workspace_bytes(3, 4096) == 12288
    assert L.pq_linear_dynamic_workspace_bytes(3, 4096, 4) == 6144 + 256
    assert L.pq_linear_dynamic_workspace_bytes(100, 128, 8) == 12800 + 512
    assert L.pq_linear_dynamic_workspace_bytes(3, 4096, 5) == 0
    assert L.pq_calibrate_workspace_bytes(256, 50) == 256 * 51 * 4
    assert L.pq_calibrate_workspace_bytes(256, 1) == 0 and L.pq_calibrate_workspace_bytes(256, 129) == 0
    assert L.pq_calibrate_zp_workspace_bytes(256, 64) == 256 * 66 * 4 and L.pq_calibrate_zp_workspace_bytes(256, 1) == 0


def test_argument_errors_launch_nothing(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)          # never dereferenced: each call fails validation first
    odd = ctypes.c_void_p(0x1008)
    nul = ctypes.c_void_p(0)
    rq = L.pq_rotate_quant
    assert rq(nul, 4, 512, 128, 0.1, p, nul) == b.PQ_ERR_NULL
    assert rq(p, 4, 512, 128, 0.1, nul, nul) == b.PQ_ERR_NULL
    assert rq(p, -1, 512, 128, 0.1, p, nul) == b.PQ_ERR_SHAPE
    assert rq(p, 4, 500, 1, 0.1, p, nul) == b.PQ_ERR_SHAPE          # K % 32
    assert rq(p, 4, 512, 96, 0.1, p, nul) == b.PQ_ERR_SHAPE         # not a power of two
    assert rq(p, 4, 1536, 1024, 0.1, p, nul) == b.PQ_ERR_SHAPE      # does not divide K
    assert rq(p, 4, 65536, 32768, 0.1, p, nul) == b.PQ_ERR_SHAPE    # too large
    assert rq(odd, 4, 512, 128, 0.1, p, nul) == b.PQ_ERR_ALIGN
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        assert rq(p, 4, 512, 128, bad, p, nul) == b.PQ_ERR_SCALE
    assert rq(p, 0, 512, 128, 0.1, p, nul) == b.PQ_OK               # empty input: no-op

    for g in (L.pq_w4a4_gemm, L.pq_w4a4_gemm_simple):
        assert g(nul, p, p, 0.1, 4, 64, 512, p, nul, nul) == b.PQ_ERR_NULL
        assert g(p, p, nul, 0.1, 4, 64, 512, p, nul, nul) == b.PQ_ERR_NULL
        assert g(p, p, p, 0.1, 4, 64, 512, nul, nul, nul) == b.PQ_ERR_NULL      # no output at all
        assert g(p, p, p, 0.1, 4, 60, 512, p, nul, nul) == b.PQ_ERR_SHAPE       # N % 16
        assert g(p, p, p, 0.1, 4, 64, 48, p, nul, nul) == b.PQ_ERR_SHAPE        # K % 32
        assert g(p, odd, p, 0.1, 4, 64, 512, p, nul, nul) == b.PQ_ERR_ALIGN
        assert g(p, p, p, -2.0, 4, 64, 512, p, nul, nul) == b.PQ_ERR_SCALE
        assert g(p, p, p, 0.1, 0, 64, 512, p, nul, nul) == b.PQ_OK

    gw = L.pq_w4a4_gemm_ws
    assert gw(nul, p, p, 0.1, 64, 64, 512, p, nul, nul, 0, nul) == b.PQ_ERR_NULL
    assert gw(p, p, p, 0.1, 64, 60, 512, p, nul, nul, 0, nul) == b.PQ_ERR_SHAPE
    assert gw(p, p, p, 0.1, 64, 64, 512, p, nul, odd, 1 << 20, nul) == b.PQ_ERR_ALIGN      # workspace: 256 bytes
    assert gw(p, p, p, 0.0, 64, 64, 512, p, nul, nul, 0, nul) == b.PQ_ERR_SCALE
    assert gw(p, p, p, 0.1, 0, 64, 512, p, nul, nul, 0, nul) == b.PQ_OK
    prev = L.pq_set_gemm_variant(5)
    try:
        assert gw(p, p, p, 0.1, 64, 64, 512, p, nul, nul, 0, nul) == b.PQ_ERR_UNSUPPORTED   # forced split, no planes
    finally:
        L.pq_set_gemm_variant(prev)

    # the widened products with scratch memory: the same checks as without, plus the workspace's alignment
    assert L.pq_w4a8_gemm_ws(p, p, p, 0.1, 64, 64, 512, p, nul, odd, 1 << 20, nul) == b.PQ_ERR_ALIGN
    assert L.pq_w4a8_gemm_ws(p, p, p, 0.1, 64, 64, 160, p, nul, nul, 0, nul) == b.PQ_ERR_SHAPE
    assert L.pq_w4a8_gemm_ws(nul, p, p, 0.1, 64, 64, 512, p, nul, nul, 0, nul) == b.PQ_ERR_NULL
    assert L.pq_gemm_dynamic_ws(p, 4, p, p, p, 64, 64, 512, p, nul, odd, 1 << 20, nul) == b.PQ_ERR_ALIGN
    assert L.pq_gemm_dynamic_ws(p, 5, p, p, p, 64, 64, 512, p, nul, nul, 0, nul) == b.PQ_ERR_SHAPE
    assert L.pq_gemm_dynamic_ws(p, 4, p, p, nul, 64, 64, 512, p, nul, nul, 0, nul) == b.PQ_ERR_NULL
    assert L.pq_w4a4_gemm_zp_ws(p, p, p, 0.1, p, 64, 64, 512, p, nul, odd, 1 << 20, nul) == b.PQ_ERR_ALIGN
    assert L.pq_w4a4_gemm_zp_ws(p, p, p, 0.1, nul, 64, 64, 512, p, nul, nul, 0, nul) == b.PQ_ERR_NULL
    assert L.pq_w4a4_gemm_zp_ws(p, p, p, 0.1, p, 64, 64, 65536, p, nul, nul, 0, nul) == b.PQ_ERR_UNSUPPORTED

    lin = L.pq_linear
    assert lin(p, p, p, 0.1, 128, 4, 64, 512, p, nul, 0, nul) == b.PQ_ERR_WORKSPACE
    assert lin(p, p, p, 0.1, 128, 4, 64, 512, p, p, 1023, nul) == b.PQ_ERR_WORKSPACE
    assert lin(p, p, p, 0.1, 128, 4, 64, 512, p, odd, 4096, nul) == b.PQ_ERR_ALIGN
    assert lin(p, p, p, 0.1, 128, 4, 64, 512, nul, p, 4096, nul) == b.PQ_ERR_NULL
    assert lin(p, p, p, 0.1, 100, 4, 64, 512, p, p, 4096, nul) == b.PQ_ERR_SHAPE
    assert lin(p, p, p, 0.0, 128, 4, 64, 512, p, p, 4096, nul) == b.PQ_ERR_SCALE
    assert lin(p, p, p, 0.1, 128, 0, 64, 512, p, nul, 0, nul) == b.PQ_OK
    prev = L.pq_set_gemm_variant(1)
    try:
        assert L.pq_w4a4_gemm(p, p, p, 0.1, 33, 64, 512, p, nul, nul) == b.PQ_ERR_UNSUPPORTED
    finally:
        L.pq_set_gemm_variant(prev)
    # the tiled kernel's accumulators carry 256 * acc: rows of 2^17 channels and more are refused, not wrapped
    assert L.pq_w4a4_gemm(p, p, p, 0.1, 40, 64, 131072, p, nul, nul) == b.PQ_ERR_UNSUPPORTED
    assert L.pq_w4a4_gemm(p, p, p, 0.1, 40, 64, 131072 + 32, p, nul, nul) == b.PQ_ERR_UNSUPPORTED    # generic kernel too
    assert gw(p, p, p, 0.1, 40, 64, 1 << 20, p, nul, ctypes.c_void_p(0x10000), 1 << 30, nul) == b.PQ_ERR_UNSUPPORTED
    # the channel steps are loaded four at a time: 16-byte alignment, as the header says
    assert L.pq_w4a4_gemm(p, p, ctypes.c_void_p(0x1004), 0.1, 4, 64, 512, p, nul, nul) == b.PQ_ERR_ALIGN
    assert lin(p, p, ctypes.c_void_p(0x1004), 0.1, 128, 4, 64, 512, p, ctypes.c_void_p(0x10000), 4096, nul) == b.PQ_ERR_ALIGN


def test_argument_errors_of_the_two_matrix_layers(b):
    """pq_linear2 and pq_linear2_f6 check both matrices before anything is enqueued (fake pointers: no GPU needed)."""
    L = b.lib()
    p, big, nul, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x10000), ctypes.c_void_p(0), ctypes.c_void_p(0x1008)
    for fn, k in ((L.pq_linear2, 512), (L.pq_linear2_f6, 512)):
        ok = dict(x=p, wa=p, sa=p, na=64, oa=p, wb=p, sb=p, nb=32, ob=p, s=0.1, h=128, m=4, k=k, ws=big, wsb=1 << 20, st=nul)

        def call(**kw):
            a = dict(ok, **kw)
            return fn(a["x"], a["wa"], a["sa"], a["na"], a["oa"], a["wb"], a["sb"], a["nb"], a["ob"], a["s"], a["h"], a["m"], a["k"],
                      a["ws"], a["wsb"], a["st"])

        assert call(m=0) == b.PQ_OK
        assert call(wb=nul) == b.PQ_ERR_NULL and call(ob=nul) == b.PQ_ERR_NULL and call(sa=nul) == b.PQ_ERR_NULL
        assert call(nb=40) == b.PQ_ERR_SHAPE and call(na=0) == b.PQ_ERR_SHAPE and call(h=100) == b.PQ_ERR_SHAPE
        assert call(ws=nul) == b.PQ_ERR_WORKSPACE and call(wsb=16) == b.PQ_ERR_WORKSPACE
        assert call(ws=odd) == b.PQ_ERR_ALIGN and call(sb=ctypes.c_void_p(0x1004)) == b.PQ_ERR_ALIGN
        assert call(s=0.0) == b.PQ_ERR_SCALE and call(s=float("nan")) == b.PQ_ERR_SCALE
    assert L.pq_linear2_f6(p, p, p, 64, p, p, p, 32, p, 0.1, 1, 4, 480, big, 1 << 20, nul) == b.PQ_ERR_SHAPE       # K % 128
    assert L.pq_linear2_f6(p, p, p, 64, p, p, p, 32, p, 0.1, 1, 4, 262144, big, 1 << 30, nul) == b.PQ_ERR_UNSUPPORTED  # sums no longer exact


def test_process_wide_switches(b):
    L = b.lib()
    assert L.pq_set_gemm_tile(99) == -2 and L.pq_set_gemm_tile(-2) == -2
    first = L.pq_set_gemm_tile(3)
    assert first in range(-1, 9)            # the environment's value at the first call, -1 unless set
    assert L.pq_set_gemm_tile(first) == 3
    assert L.pq_set_gemm_f6_tile(5) == -2 and L.pq_set_gemm_f6_tile(0) == -2
    first = L.pq_set_gemm_f6_tile(3)
    assert first in (-1, 2, 3, 4)
    assert L.pq_set_gemm_f6_tile(first) == 3


def test_noalloc_size_checks_need_no_gpu(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)
    nul = ctypes.c_void_p(0)
    limit = L.pq_linear_noalloc_max_bytes()
    assert limit == 32 << 20
    na = L.pq_linear_noalloc
    assert na(p, p, p, 0.1, 1, 2048, 64, 2 * (limit // 2048) + 64, p, nul) == b.PQ_ERR_WORKSPACE
    assert na(p, p, p, 0.1, 1, 1 << 40, 64, 64, p, nul) == b.PQ_ERR_WORKSPACE
    assert na(p, p, p, 0.1, 1, 4, 64, 1 << 40, p, nul) == b.PQ_ERR_WORKSPACE
    assert na(p, p, p, 0.1, 1, 4, 60, 64, p, nul) == b.PQ_ERR_SHAPE
    assert na(p, p, p, 0.1, 1, 4, 64, 48, p, nul) == b.PQ_ERR_SHAPE
    assert na(p, p, p, 0.1, 1, 0, 64, 64, p, nul) == b.PQ_OK


def test_argument_errors_of_the_f6_probes(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    nul = ctypes.c_void_p(0)
    assert L.pq_probe_f6_product(nul, p, 64, p, nul) == b.PQ_ERR_NULL
    assert L.pq_probe_f6_product(p, p, 64, nul, nul) == b.PQ_ERR_NULL
    assert L.pq_probe_f6_product(odd, p, 64, p, nul) == b.PQ_ERR_ALIGN
    assert L.pq_probe_f6_product(p, p, 96, p, nul) == b.PQ_ERR_SHAPE          # K % 64
    assert L.pq_probe_f6_product(p, p, 262144, p, nul) == b.PQ_ERR_SHAPE      # sums could pass 2^24
    assert L.pq_probe_mfma_f6(nul, 64, 1, 1, p, nul) == b.PQ_ERR_NULL
    assert L.pq_probe_mfma_f6(ctypes.c_void_p(0x1010), 64, 1, 1, p, nul) == b.PQ_ERR_ALIGN    # 32 bytes
    assert L.pq_probe_mfma_f6(p, 48, 1, 1, p, nul) == b.PQ_ERR_SHAPE
    assert L.pq_probe_mfma_f6(p, 64, 1, 0, p, nul) == b.PQ_ERR_SHAPE


def test_argument_errors_of_the_f6_product(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    nul = ctypes.c_void_p(0)
    assert L.pq_f6_tiles_bytes(32, 128) == 3072 and L.pq_f6_tiles_bytes(33, 256) == 2 * 2 * 3072
    assert L.pq_f6_tiles_bytes(2048, 4096) == 2048 * 4096 * 3 // 4
    assert L.pq_f6_tiles_bytes(32, 64) == 0 and L.pq_f6_tiles_bytes(0, 128) == 0
    rp = L.pq_repack_f6
    assert rp(nul, 32, 128, p, nul) == b.PQ_ERR_NULL and rp(p, 32, 128, nul, nul) == b.PQ_ERR_NULL
    assert rp(p, 32, 64, p, nul) == b.PQ_ERR_SHAPE and rp(p, -1, 128, p, nul) == b.PQ_ERR_SHAPE
    assert rp(odd, 32, 128, p, nul) == b.PQ_ERR_ALIGN
    assert rp(p, 0, 128, p, nul) == b.PQ_OK
    assert rp(p, 32, 262144, p, nul) == b.PQ_ERR_UNSUPPORTED         # sums could pass 2^24
    assert L.pq_linear_f6_workspace_bytes(2048, 4096, 1) == 2048 * 4096 * 3 // 4
    assert L.pq_linear_f6_workspace_bytes(2048, 4096, 128) == 2048 * 4096 * 3 // 4
    assert L.pq_linear_f6_workspace_bytes(2048, 4096, 4096) == 2048 * 4096 * 3 // 4 + 2048 * 2048   # codes as well
    assert L.pq_linear_f6_workspace_bytes(3, 128, 0) == 3072 and L.pq_linear_f6_workspace_bytes(3, 96, 1) == 0
    rq6 = L.pq_rotate_quant_f6
    assert rq6(nul, 32, 128, 1, 0.1, p, nul, nul) == b.PQ_ERR_NULL and rq6(p, 32, 128, 1, 0.1, nul, nul, nul) == b.PQ_ERR_NULL
    assert rq6(p, 32, 96, 1, 0.1, p, nul, nul) == b.PQ_ERR_SHAPE and rq6(p, 32, 256, 48, 0.1, p, nul, nul) == b.PQ_ERR_SHAPE
    assert rq6(p, 32, 128, 1, 0.1, p, odd, nul) == b.PQ_ERR_ALIGN and rq6(p, 32, 128, 1, -1.0, p, nul, nul) == b.PQ_ERR_SCALE
    assert rq6(p, 32, 2048, 1024, 0.1, p, nul, nul) == b.PQ_ERR_UNSUPPORTED          # blocks beyond 512 channels
    assert rq6(p, 0, 128, 1, 0.1, p, nul, nul) == b.PQ_OK
    lf = L.pq_linear_f6
    p256 = ctypes.c_void_p(0x10000)
    assert lf(p, p, p, 0.1, 1, 32, 16, 128, p, nul, 0, nul) == b.PQ_ERR_WORKSPACE
    assert lf(p, p, p, 0.1, 1, 32, 16, 128, p, p256, 100, nul) == b.PQ_ERR_WORKSPACE
    assert lf(p, p, p, 0.1, 1, 32, 16, 128, p, odd, 1 << 20, nul) == b.PQ_ERR_ALIGN
    assert lf(nul, p, p, 0.1, 1, 32, 16, 128, p, p256, 1 << 20, nul) == b.PQ_ERR_NULL
    assert lf(p, p, p, 0.1, 96, 32, 16, 128, p, p256, 1 << 20, nul) == b.PQ_ERR_SHAPE
    assert lf(p, p, p, 0.1, 1, 32, 16, 64, p, p256, 1 << 20, nul) == b.PQ_ERR_SHAPE
    assert lf(p, p, p, -1.0, 1, 32, 16, 128, p, p256, 1 << 20, nul) == b.PQ_ERR_SCALE
    assert lf(p, p, p, 0.1, 1, 0, 16, 128, p, nul, 0, nul) == b.PQ_OK
    g = L.pq_w4a4_gemm_f6
    assert g(nul, p, p, 0.1, 32, 16, 128, p, nul, nul) == b.PQ_ERR_NULL
    assert g(p, p, p, 0.1, 32, 16, 128, nul, nul, nul) == b.PQ_ERR_NULL
    assert g(p, p, p, 0.1, 32, 16, 160, p, nul, nul) == b.PQ_ERR_SHAPE       # K % 128
    assert g(p, p, p, 0.1, 32, 20, 128, p, nul, nul) == b.PQ_ERR_SHAPE       # N % 16
    assert g(p, odd, p, 0.1, 32, 16, 128, p, nul, nul) == b.PQ_ERR_ALIGN
    assert g(p, p, p, float("nan"), 32, 16, 128, p, nul, nul) == b.PQ_ERR_SCALE
    assert g(p, p, p, 0.1, 0, 16, 128, p, nul, nul) == b.PQ_OK


def test_argument_errors_of_the_widened_calls(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)          # never dereferenced: each call fails validation first
    p256 = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x1008)
    nul = ctypes.c_void_p(0)
    E = b
    # 8-bit static
    assert L.pq_rotate_quant8(p, 4, 160, 1, 0.1, p, nul) == E.PQ_ERR_SHAPE              # K % 128
    assert L.pq_rotate_quant8(p, 4, 256, 1, 0.1, nul, nul) == E.PQ_ERR_NULL
    assert L.pq_rotate_quant8(p, 4, 256, 1, -0.1, p, nul) == E.PQ_ERR_SCALE
    assert L.pq_rotate_quant8(p, 0, 256, 1, 0.1, p, nul) == E.PQ_OK
    assert L.pq_w4a8_gemm(p, p, p, 0.1, 4, 64, 160, p, nul, nul) == E.PQ_ERR_SHAPE
    assert L.pq_w4a8_gemm(p, p, p, 0.1, 4, 64, 256, nul, nul, nul) == E.PQ_ERR_NULL
    assert L.pq_w4a8_gemm(p, p, p, 0.1, 40, 64, 131072, p, nul, nul) == E.PQ_ERR_UNSUPPORTED   # K > 65536
    assert L.pq_linear_w4a8(p, p, p, 0.1, 128, 4, 64, 256, p, p256, 512, nul) == E.PQ_ERR_WORKSPACE
    assert L.pq_linear_w4a8(p, p, p, 0.1, 128, 4, 64, 256, p, odd, 4096, nul) == E.PQ_ERR_ALIGN
    assert L.pq_linear_w4a8(p, p, p, 0.1, 128, 0, 64, 256, p, nul, 0, nul) == E.PQ_OK
    # per-token dynamic
    rqd = L.pq_rotate_quant_dynamic
    assert rqd(p, 4, 256, 1, 1.0, 4, p, nul, nul) == E.PQ_ERR_NULL                       # no place for the steps
    assert rqd(p, 4, 256, 1, 1.0, 6, p, p, nul) == E.PQ_ERR_SHAPE
    assert rqd(p, 4, 256, 1, 0.0, 4, p, p, nul) == E.PQ_ERR_SCALE
    assert rqd(p, 4, 256, 1, 1.25, 4, p, p, nul) == E.PQ_ERR_SCALE
    assert rqd(p, 4, 32768 + 128, 1, 1.0, 4, p, p, nul) == E.PQ_ERR_UNSUPPORTED
    assert rqd(p, 4, 256, 1, 1.0, 4, p, ctypes.c_void_p(0x1002), nul) == E.PQ_ERR_ALIGN
    assert L.pq_gemm_dynamic(p, 4, p, p, nul, 4, 64, 256, p, nul, nul) == E.PQ_ERR_NULL
    assert L.pq_gemm_dynamic(p, 3, p, p, p, 4, 64, 256, p, nul, nul) == E.PQ_ERR_SHAPE
    assert L.pq_linear_dynamic(p, p, p, 1.0, 1, 4, 4, 64, 256, p, p256, 512, nul) == E.PQ_ERR_WORKSPACE   # needs 512 + 256
    assert L.pq_linear_dynamic(p, p, p, 1.0, 1, 4, 0, 64, 256, p, nul, 0, nul) == E.PQ_OK
    # attention side
    rh = L.pq_rotate_quant_heads
    assert rh(p, 4, 8, 48, 1, p, p, nul) == E.PQ_ERR_SHAPE                               # head_dim not a power of two
    assert rh(p, 4, 8, 16, 1, p, p, nul) == E.PQ_ERR_SHAPE                               # head_dim < 32
    assert rh(p, 4, 0, 128, 1, p, p, nul) == E.PQ_ERR_SHAPE
    assert rh(p, 4, 8, 128, 1, nul, p, nul) == E.PQ_ERR_NULL
    assert rh(p, 4, 8, 128, 1, ctypes.c_void_p(0x1001), p, nul) == E.PQ_ERR_ALIGN
    assert rh(p, 0, 8, 128, 1, p, p, nul) == E.PQ_OK
    assert L.pq_rotate_f16(p, 4, 256, 1, p, nul) == E.PQ_ERR_SHAPE                       # nothing to rotate
    assert L.pq_rotate_f16(p, 4, 256, 96, p, nul) == E.PQ_ERR_SHAPE
    assert L.pq_rotate_f16(p, 4, 256, 128, nul, nul) == E.PQ_ERR_NULL
    # fused producers
    assert L.pq_silu_mul_rotate_quant(p, nul, 4, 256, 128, 0.1, p, nul) == E.PQ_ERR_NULL
    assert L.pq_silu_mul_rotate_quant(p, p, 4, 250, 1, 0.1, p, nul) == E.PQ_ERR_SHAPE
    assert L.pq_silu_mul_rotate_quant(p, odd, 4, 256, 128, 0.1, p, nul) == E.PQ_ERR_ALIGN
    assert L.pq_rmsnorm_quant(p, 4, 256, -1e-6, 0.1, p, nul) == E.PQ_ERR_SCALE
    assert L.pq_rmsnorm_quant(p, 4, 65536, 1e-6, 0.1, p, nul) == E.PQ_ERR_UNSUPPORTED
    assert L.pq_rmsnorm_quant(p, 0, 256, 1e-6, 0.1, p, nul) == E.PQ_OK
    # calibration
    cal = L.pq_calibrate_static
    assert cal(p, 0, 256, 1, 4, 8, 0.5, p, p256, 1 << 20, nul) == E.PQ_ERR_SHAPE          # no tokens
    assert cal(p, 4, 256, 1, 4, 1, 0.5, p, p256, 1 << 20, nul) == E.PQ_ERR_SHAPE
    assert cal(p, 4, 256, 1, 4, 8, 1.0, p, p256, 1 << 20, nul) == E.PQ_ERR_SCALE
    assert cal(p, 4, 256, 1, 4, 8, 0.5, p, p256, 16, nul) == E.PQ_ERR_WORKSPACE
    assert cal(p, 4, 256, 1, 4, 8, 0.5, nul, p256, 1 << 20, nul) == E.PQ_ERR_NULL
    assert cal(p, 4, 65536, 1, 4, 8, 0.5, p, p256, 1 << 20, nul) == E.PQ_ERR_UNSUPPORTED


def test_argument_errors_of_the_probes(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)          # never dereferenced: each call fails validation first
    odd = ctypes.c_void_p(0x1008)
    nul = ctypes.c_void_p(0)
    assert L.pq_probe_mfma_i8(nul, 1024, 10, 256, p, nul) == b.PQ_ERR_NULL
    assert L.pq_probe_mfma_i8(p, 1024, 10, 256, nul, nul) == b.PQ_ERR_NULL
    assert L.pq_probe_mfma_i8(odd, 1024, 10, 256, p, nul) == b.PQ_ERR_ALIGN
    assert L.pq_probe_mfma_i8(p, 1000, 10, 256, p, nul) == b.PQ_ERR_SHAPE          # bytes % 16
    assert L.pq_probe_mfma_i8(p, 1024, -1, 256, p, nul) == b.PQ_ERR_SHAPE
    assert L.pq_probe_mfma_i8(p, 1024, 10, 0, p, nul) == b.PQ_ERR_SHAPE
    assert L.pq_probe_stream_read(nul, 1024, p, nul) == b.PQ_ERR_NULL
    assert L.pq_probe_stream_read(odd, 1024, p, nul) == b.PQ_ERR_ALIGN
    assert L.pq_probe_stream_read(p, 8, p, nul) == b.PQ_ERR_SHAPE
