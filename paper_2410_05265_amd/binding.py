"""ctypes binding of libpq.so: argument marshalling only.

Every step of the layer runs in the HIP kernels behind the C ABI declared in
include/pq.h; torch is used here for device memory and the current stream, nothing else.
There is no CPU fallback: if the library has not been built, loading raises.
"""

from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpq.so")

PQ_OK, PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_ALIGN, PQ_ERR_SCALE, PQ_ERR_WORKSPACE, PQ_ERR_HIP, PQ_ERR_UNSUPPORTED = range(8)

_i64, _i32, _f32, _vp, _sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t

# symbol -> (restype, argtypes); mirrors include/pq.h
SIGNATURES = {
    "pq_version": (ctypes.c_int, []),
    "pq_status_str": (ctypes.c_char_p, [ctypes.c_int]),
    "pq_rotate_quant": (ctypes.c_int, [_vp, _i64, _i64, _i32, _f32, _vp, _vp]),
    "pq_w4a4_gemm": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i64, _i64, _i64, _vp, _vp, _vp]),
    "pq_w4a4_gemm_simple": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i64, _i64, _i64, _vp, _vp, _vp]),
    "pq_linear_workspace_bytes": (_sz, [_i64, _i64]),
    "pq_linear_workspace_bytes_split": (_sz, [_i64, _i64, _i64]),
    "pq_w4a4_gemm_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "pq_w4a4_gemm_ws": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i64, _i64, _i64, _vp, _vp, _vp, _sz, _vp]),
    "pq_linear": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i32, _i64, _i64, _i64, _vp, _vp, _sz, _vp]),
    "pq_linear2": (ctypes.c_int, [_vp, _vp, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _f32, _i32, _i64, _i64, _vp, _sz, _vp]),
    "pq_prepacked_bytes": (_sz, [_i64, _i64]),
    "pq_prepack_weights": (ctypes.c_int, [_vp, _i64, _i64, _vp, _vp]),
    "pq_linear_prepacked": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i32, _i64, _i64, _i64, _vp, _vp, _sz, _vp]),
    "pq_linear2_f6": (ctypes.c_int, [_vp, _vp, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _f32, _i32, _i64, _i64, _vp, _sz, _vp]),
    "pq_linear_noalloc_max_bytes": (_sz, []),
    "pq_linear_noalloc": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i32, _i64, _i64, _i64, _vp, _vp]),
    "pq_set_gemm_variant": (ctypes.c_int, [ctypes.c_int]),
    "pq_set_gemm_tile": (ctypes.c_int, [ctypes.c_int]),
    "pq_set_gemm_f6_tile": (ctypes.c_int, [ctypes.c_int]),
    "pq_probe_mfma_i8": (ctypes.c_int, [_vp, _i64, _i64, _i32, _vp, _vp]),
    "pq_probe_stream_read": (ctypes.c_int, [_vp, _i64, _vp, _vp]),
    "pq_probe_mfma_f6": (ctypes.c_int, [_vp, _i64, _i64, _i32, _vp, _vp]),
    "pq_f6_tiles_bytes": (_sz, [_i64, _i64]),
    "pq_repack_f6": (ctypes.c_int, [_vp, _i64, _i64, _vp, _vp]),
    "pq_w4a4_gemm_f6": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i64, _i64, _i64, _vp, _vp, _vp]),
    "pq_linear_f6_workspace_bytes": (_sz, [_i64, _i64, _i32]),
    "pq_rotate_quant_f6": (ctypes.c_int, [_vp, _i64, _i64, _i32, _f32, _vp, _vp, _vp]),
    "pq_linear_f6": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i32, _i64, _i64, _i64, _vp, _vp, _sz, _vp]),
    "pq_probe_f6_product": (ctypes.c_int, [_vp, _vp, _i64, _vp, _vp]),
    "pq_rotate_quant8": (ctypes.c_int, [_vp, _i64, _i64, _i32, _f32, _vp, _vp]),
    "pq_w4a8_gemm": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i64, _i64, _i64, _vp, _vp, _vp]),
    "pq_w4a8_gemm_ws": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i64, _i64, _i64, _vp, _vp, _vp, _sz, _vp]),
    "pq_gemm_workspace_bytes": (_sz, [_i64, _i64, _i64, _i32]),
    "pq_linear_w4a8_workspace_bytes_split": (_sz, [_i64, _i64, _i64]),
    "pq_linear_w4a8_workspace_bytes": (_sz, [_i64, _i64]),
    "pq_linear_w4a8": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i32, _i64, _i64, _i64, _vp, _vp, _sz, _vp]),
    "pq_rotate_quant_dynamic": (ctypes.c_int, [_vp, _i64, _i64, _i32, _f32, _i32, _vp, _vp, _vp]),
    "pq_gemm_dynamic": (ctypes.c_int, [_vp, _i32, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp]),
    "pq_gemm_dynamic_ws": (ctypes.c_int, [_vp, _i32, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _sz, _vp]),
    "pq_linear_dynamic_workspace_bytes_split": (_sz, [_i64, _i64, _i64, _i32]),
    "pq_linear_dynamic_workspace_bytes": (_sz, [_i64, _i64, _i32]),
    "pq_linear_dynamic": (ctypes.c_int, [_vp, _vp, _vp, _f32, _i32, _i32, _i64, _i64, _i64, _vp, _vp, _sz, _vp]),
    "pq_rotate_quant_heads": (ctypes.c_int, [_vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp]),
    "pq_rotate_quant_groups": (ctypes.c_int, [_vp, _i64, _i32, _i32, _i32, _i32, _f32, _vp, _vp, _vp]),
    "pq_rotate_f16": (ctypes.c_int, [_vp, _i64, _i64, _i32, _vp, _vp]),
    "pq_silu_mul_rotate_quant": (ctypes.c_int, [_vp, _vp, _i64, _i64, _i32, _f32, _vp, _vp]),
    "pq_rmsnorm_quant": (ctypes.c_int, [_vp, _i64, _i64, _f32, _f32, _vp, _vp]),
    "pq_rotate_quant_zp": (ctypes.c_int, [_vp, _i64, _i64, _i32, _f32, _i32, _vp, _vp]),
    "pq_zero_point_correction": (ctypes.c_int, [_vp, _i64, _i64, _i32, _vp, _vp]),
    "pq_w4a4_gemm_zp": (ctypes.c_int, [_vp, _vp, _vp, _f32, _vp, _i64, _i64, _i64, _vp, _vp, _vp]),
    "pq_w4a4_gemm_zp_ws": (ctypes.c_int, [_vp, _vp, _vp, _f32, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _sz, _vp]),
    "pq_calibrate_workspace_bytes": (_sz, [_i64, _i32]),
    "pq_calibrate_zp_workspace_bytes": (_sz, [_i64, _i32]),
    "pq_calibrate_static_zp": (ctypes.c_int, [_vp, _i64, _i64, _i32, _i32, _i32, _f32, _f32, _vp, _vp, _sz, _vp]),
    "pq_calibrate_static": (ctypes.c_int, [_vp, _i64, _i64, _i32, _i32, _i32, _f32, _vp, _vp, _sz, _vp]),
}

_lib = None


class PQError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_str(status)))


def lib() -> ctypes.CDLL:
    """The loaded library; raises if libpq.so is missing (build it with build.build_lib())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: the HIP library is not built (python -m paper_2410_05265_amd.build)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().pq_status_str(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _ws_args(workspace):
    """(pointer, bytes) of an optional uint8 scratch tensor."""
    if workspace is None:
        return None, 0
    _dev(workspace, torch.uint8, "workspace")
    return _ptr(workspace), workspace.numel()


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != PQ_OK:
        raise PQError(rc, where)


def _dev(t: torch.Tensor, dtype, what: str):
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous %s tensor on the GPU" % (what, dtype))


def pq_rotate_quant(x: torch.Tensor, had_block: int, act_scale: float, out: torch.Tensor | None = None):
    """x fp16 [M,K] -> packed codes uint8 [M,K/2]."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if out is None:
        out = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    _check(lib().pq_rotate_quant(_ptr(x), M, K, int(had_block), float(act_scale), _ptr(out), _stream()),
           "pq_rotate_quant")
    return out


def _gemm(fn, name, xq, wq, w_scale, act_scale, want_out, want_acc, out, acc):
    _dev(xq, torch.uint8, "xq")
    _dev(wq, torch.uint8, "wq")
    _dev(w_scale, torch.float32, "w_scale")
    M, K = xq.shape[0], xq.shape[1] * 2
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or w_scale.numel() != N:
        raise ValueError("shape mismatch")
    if want_out and out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    _check(fn(_ptr(xq), _ptr(wq), _ptr(w_scale), float(act_scale), M, N, K, _ptr(out), _ptr(acc), _stream()), name)
    return out, acc


def pq_w4a4_gemm(xq, wq, w_scale, act_scale, want_out=True, want_acc=False, out=None, acc=None):
    """packed codes [M,K/2] x packed weights [N,K/2] -> (out fp16 [M,N] | None, acc int32 [M,N] | None)."""
    return _gemm(lib().pq_w4a4_gemm, "pq_w4a4_gemm", xq, wq, w_scale, act_scale, want_out, want_acc, out, acc)


def pq_w4a4_gemm_simple(xq, wq, w_scale, act_scale, want_out=True, want_acc=False, out=None, acc=None):
    return _gemm(lib().pq_w4a4_gemm_simple, "pq_w4a4_gemm_simple", xq, wq, w_scale, act_scale, want_out, want_acc,
                 out, acc)


def pq_w4a4_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().pq_w4a4_gemm_workspace_bytes(M, N, K))


def pq_w4a4_gemm_ws(xq, wq, w_scale, act_scale, workspace, want_out=True, want_acc=False, out=None, acc=None):
    """pq_w4a4_gemm with scratch memory (uint8 device tensor or None) for the split-K launch."""
    if workspace is not None:
        _dev(workspace, torch.uint8, "workspace")

    def fn(a, b, c, d, M, N, K, o, ac, st):
        return lib().pq_w4a4_gemm_ws(a, b, c, d, M, N, K, o, ac, _ptr(workspace),
                                     0 if workspace is None else workspace.numel(), st)
    return _gemm(fn, "pq_w4a4_gemm_ws", xq, wq, w_scale, act_scale, want_out, want_acc, out, acc)


def pq_linear_workspace_bytes_split(M: int, N: int, K: int) -> int:
    return int(lib().pq_linear_workspace_bytes_split(M, N, K))


def pq_linear_workspace_bytes(M: int, K: int) -> int:
    return int(lib().pq_linear_workspace_bytes(M, K))


def pq_linear(x, wq, w_scale, act_scale, had_block, out=None, workspace=None):
    """The whole layer.  Returns (out fp16 [M,N], workspace uint8 holding the packed codes)."""
    _dev(x, torch.float16, "x")
    _dev(wq, torch.uint8, "wq")
    _dev(w_scale, torch.float32, "w_scale")
    M, K = x.shape
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or w_scale.numel() != N:
        raise ValueError("shape mismatch")
    need = pq_linear_workspace_bytes(M, K)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().pq_linear(_ptr(x), _ptr(wq), _ptr(w_scale), float(act_scale), int(had_block), M, N, K, _ptr(out),
                           _ptr(workspace), workspace.numel(), _stream()), "pq_linear")
    return out, workspace


def pq_linear2(x, wq_a, w_scale_a, wq_b, w_scale_b, act_scale, had_block, out_a=None, out_b=None, workspace=None):
    """Two layers on the same tokens (gate and up).  Returns (out_a, out_b, workspace)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    for w, s in ((wq_a, w_scale_a), (wq_b, w_scale_b)):
        _dev(w, torch.uint8, "wq")
        _dev(s, torch.float32, "w_scale")
        if w.shape[1] * 2 != K or s.numel() != w.shape[0]:
            raise ValueError("shape mismatch")
    Na, Nb = wq_a.shape[0], wq_b.shape[0]
    if workspace is None:
        workspace = torch.empty((max(pq_linear_workspace_bytes(M, K), 256),), dtype=torch.uint8, device=x.device)
    if out_a is None:
        out_a = torch.empty((M, Na), dtype=torch.float16, device=x.device)
    if out_b is None:
        out_b = torch.empty((M, Nb), dtype=torch.float16, device=x.device)
    _check(lib().pq_linear2(_ptr(x), _ptr(wq_a), _ptr(w_scale_a), Na, _ptr(out_a), _ptr(wq_b), _ptr(w_scale_b), Nb,
                            _ptr(out_b), float(act_scale), int(had_block), M, K, _ptr(workspace), workspace.numel(),
                            _stream()), "pq_linear2")
    return out_a, out_b, workspace


def pq_linear2_f6(x, w_tiles_a, w_scale_a, w_tiles_b, w_scale_b, act_scale, had_block, out_a=None, out_b=None, workspace=None):
    """pq_linear2 with prepacked weights (pq_repack_f6).  Returns (out_a, out_b, workspace holding the tiles of Xq)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    for s in (w_scale_a, w_scale_b):
        _dev(s, torch.float32, "w_scale")
    Na, Nb = w_scale_a.numel(), w_scale_b.numel()
    if workspace is None:
        workspace = torch.empty((max(pq_linear_f6_workspace_bytes(M, K, had_block), 256),), dtype=torch.uint8, device=x.device)
    if out_a is None:
        out_a = torch.empty((M, Na), dtype=torch.float16, device=x.device)
    if out_b is None:
        out_b = torch.empty((M, Nb), dtype=torch.float16, device=x.device)
    _check(lib().pq_linear2_f6(_ptr(x), _ptr(w_tiles_a), _ptr(w_scale_a), Na, _ptr(out_a), _ptr(w_tiles_b), _ptr(w_scale_b), Nb,
                               _ptr(out_b), float(act_scale), int(had_block), M, K, _ptr(workspace), workspace.numel(),
                               _stream()), "pq_linear2_f6")
    return out_a, out_b, workspace


def pq_prepacked_bytes(N: int, K: int) -> int:
    return int(lib().pq_prepacked_bytes(N, K))


def pq_prepack_weights(wq, out=None):
    """pq_repack_f6 on a weight matrix, under its other name.  wq uint8 [N,K/2] -> tiles."""
    _dev(wq, torch.uint8, "wq")
    N, K = wq.shape[0], wq.shape[1] * 2
    if out is None:
        out = torch.empty((pq_prepacked_bytes(N, K),), dtype=torch.uint8, device=wq.device)
    _check(lib().pq_prepack_weights(_ptr(wq), N, K, _ptr(out), _stream()), "pq_prepack_weights")
    return out


def pq_linear_prepacked(x, wq_tiled, w_scale, act_scale, had_block, out=None, workspace=None):
    """pq_linear_f6 under its other name.  Returns (out, workspace)."""
    _dev(x, torch.float16, "x")
    _dev(w_scale, torch.float32, "w_scale")
    M, K = x.shape
    N = w_scale.numel()
    if workspace is None:
        workspace = torch.empty((max(pq_linear_f6_workspace_bytes(M, K, had_block), 256),), dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().pq_linear_prepacked(_ptr(x), _ptr(wq_tiled), _ptr(w_scale), float(act_scale), int(had_block), M, N, K, _ptr(out),
                                     _ptr(workspace), workspace.numel(), _stream()), "pq_linear_prepacked")
    return out, workspace


def pq_linear_noalloc_max_bytes() -> int:
    return int(lib().pq_linear_noalloc_max_bytes())


def pq_linear_noalloc(x, wq, w_scale, act_scale, had_block, out):
    """pq_linear with the library's built-in scratch array; `out` fp16 [M,N] is the caller's (nothing is allocated)."""
    _dev(x, torch.float16, "x")
    _dev(wq, torch.uint8, "wq")
    _dev(w_scale, torch.float32, "w_scale")
    _dev(out, torch.float16, "out")
    M, K = x.shape
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or w_scale.numel() != N or tuple(out.shape) != (M, N):
        raise ValueError("shape mismatch")
    _check(lib().pq_linear_noalloc(_ptr(x), _ptr(wq), _ptr(w_scale), float(act_scale), int(had_block), M, N, K,
                                   _ptr(out), _stream()), "pq_linear_noalloc")
    return out


def pq_rotate_quant8(x: torch.Tensor, had_block: int, act_scale: float, out: torch.Tensor | None = None):
    """x fp16 [M,K] -> 8-bit codes int8 [M,K] in the grouped (even-then-odd per 32 channels) layout."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if out is None:
        out = torch.empty((M, K), dtype=torch.int8, device=x.device)
    _check(lib().pq_rotate_quant8(_ptr(x), M, K, int(had_block), float(act_scale), _ptr(out), _stream()),
           "pq_rotate_quant8")
    return out


def pq_w4a8_gemm(xq8, wq, w_scale, act_scale, want_out=True, want_acc=False, out=None, acc=None, workspace=None):
    """grouped int8 codes [M,K] x packed weights [N,K/2] -> (out fp16 | None, acc int32 | None).
    With `workspace` (uint8 scratch) the call is pq_w4a8_gemm_ws."""
    _dev(xq8, torch.int8, "xq8")
    _dev(wq, torch.uint8, "wq")
    _dev(w_scale, torch.float32, "w_scale")
    M, K = xq8.shape
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or w_scale.numel() != N:
        raise ValueError("shape mismatch")
    if want_out and out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq8.device)
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=xq8.device)
    if workspace is None:
        _check(lib().pq_w4a8_gemm(_ptr(xq8), _ptr(wq), _ptr(w_scale), float(act_scale), M, N, K, _ptr(out), _ptr(acc),
                                  _stream()), "pq_w4a8_gemm")
    else:
        _check(lib().pq_w4a8_gemm_ws(_ptr(xq8), _ptr(wq), _ptr(w_scale), float(act_scale), M, N, K, _ptr(out),
                                     _ptr(acc), *_ws_args(workspace), _stream()), "pq_w4a8_gemm_ws")
    return out, acc


def pq_w4a8_gemm_ws(xq8, wq, w_scale, act_scale, workspace, **kw):
    return pq_w4a8_gemm(xq8, wq, w_scale, act_scale, workspace=workspace, **kw)


def pq_gemm_workspace_bytes(M: int, N: int, K: int, act_bits: int) -> int:
    return int(lib().pq_gemm_workspace_bytes(M, N, K, int(act_bits)))


def pq_linear_w4a8_workspace_bytes_split(M: int, N: int, K: int) -> int:
    return int(lib().pq_linear_w4a8_workspace_bytes_split(M, N, K))


def pq_linear_w4a8_workspace_bytes(M: int, K: int) -> int:
    return int(lib().pq_linear_w4a8_workspace_bytes(M, K))


def pq_linear_w4a8(x, wq, w_scale, act_scale, had_block, out=None, workspace=None):
    """The whole W4A8 layer.  Returns (out fp16 [M,N], workspace uint8 holding the grouped int8 codes)."""
    _dev(x, torch.float16, "x")
    _dev(wq, torch.uint8, "wq")
    _dev(w_scale, torch.float32, "w_scale")
    M, K = x.shape
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or w_scale.numel() != N:
        raise ValueError("shape mismatch")
    need = pq_linear_w4a8_workspace_bytes(M, K)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().pq_linear_w4a8(_ptr(x), _ptr(wq), _ptr(w_scale), float(act_scale), int(had_block), M, N, K,
                                _ptr(out), _ptr(workspace), workspace.numel(), _stream()), "pq_linear_w4a8")
    return out, workspace


def pq_rotate_quant_dynamic(x, had_block: int, clip: float = 1.0, bits: int = 4, out=None, row_scale=None):
    """x fp16 [M,K] -> (codes: uint8 [M,K/2] packed (bits=4) or int8 [M,K] grouped (bits=8), row steps fp32 [M])."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if out is None:
        out = (torch.empty((M, K), dtype=torch.int8, device=x.device) if bits == 8
               else torch.empty((M, K // 2), dtype=torch.uint8, device=x.device))
    if row_scale is None:
        row_scale = torch.empty((max(M, 1),), dtype=torch.float32, device=x.device)[:M]
    _check(lib().pq_rotate_quant_dynamic(_ptr(x), M, K, int(had_block), float(clip), int(bits), _ptr(out),
                                         _ptr(row_scale), _stream()), "pq_rotate_quant_dynamic")
    return out, row_scale


def pq_gemm_dynamic(xq, bits, wq, w_scale, row_scale, want_out=True, want_acc=False, out=None, acc=None,
                    workspace=None):
    """codes x packed weights with per-token steps -> (out fp16 | None, acc int32 | None).
    With `workspace` (uint8 scratch) the call is pq_gemm_dynamic_ws."""
    _dev(xq, torch.int8 if bits == 8 else torch.uint8, "xq")
    _dev(wq, torch.uint8, "wq")
    _dev(w_scale, torch.float32, "w_scale")
    _dev(row_scale, torch.float32, "row_scale")
    M, K = xq.shape[0], xq.shape[1] * (1 if bits == 8 else 2)
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or w_scale.numel() != N or row_scale.numel() != M:
        raise ValueError("shape mismatch")
    if want_out and out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    if workspace is None:
        _check(lib().pq_gemm_dynamic(_ptr(xq), int(bits), _ptr(wq), _ptr(w_scale), _ptr(row_scale), M, N, K, _ptr(out),
                                     _ptr(acc), _stream()), "pq_gemm_dynamic")
    else:
        _check(lib().pq_gemm_dynamic_ws(_ptr(xq), int(bits), _ptr(wq), _ptr(w_scale), _ptr(row_scale), M, N, K,
                                        _ptr(out), _ptr(acc), *_ws_args(workspace), _stream()), "pq_gemm_dynamic_ws")
    return out, acc


def pq_gemm_dynamic_ws(xq, bits, wq, w_scale, row_scale, workspace, **kw):
    return pq_gemm_dynamic(xq, bits, wq, w_scale, row_scale, workspace=workspace, **kw)


def pq_linear_dynamic_workspace_bytes_split(M: int, N: int, K: int, bits: int = 4) -> int:
    return int(lib().pq_linear_dynamic_workspace_bytes_split(M, N, K, int(bits)))


def pq_linear_dynamic_workspace_bytes(M: int, K: int, bits: int = 4) -> int:
    return int(lib().pq_linear_dynamic_workspace_bytes(M, K, int(bits)))


def pq_linear_dynamic(x, wq, w_scale, had_block, clip: float = 1.0, bits: int = 4, out=None, workspace=None):
    """The whole per-token dynamic layer.  Returns (out fp16 [M,N], workspace uint8: codes, then row steps)."""
    _dev(x, torch.float16, "x")
    _dev(wq, torch.uint8, "wq")
    _dev(w_scale, torch.float32, "w_scale")
    M, K = x.shape
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or w_scale.numel() != N:
        raise ValueError("shape mismatch")
    need = pq_linear_dynamic_workspace_bytes(M, K, bits)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().pq_linear_dynamic(_ptr(x), _ptr(wq), _ptr(w_scale), float(clip), int(had_block), int(bits), M, N, K,
                                   _ptr(out), _ptr(workspace), workspace.numel(), _stream()), "pq_linear_dynamic")
    return out, workspace


def pq_rotate_quant_heads(x, n_heads: int, rotate: bool, head_scale, out=None):
    """x fp16 [T, n_heads*head_dim], head_scale fp32 [n_heads] -> packed codes uint8 [T, n_heads*head_dim/2]."""
    _dev(x, torch.float16, "x")
    _dev(head_scale, torch.float32, "head_scale")
    T, C = x.shape
    if C % n_heads or head_scale.numel() != n_heads:
        raise ValueError("shape mismatch")
    if out is None:
        out = torch.empty((T, C // 2), dtype=torch.uint8, device=x.device)
    _check(lib().pq_rotate_quant_heads(_ptr(x), T, int(n_heads), C // n_heads, int(bool(rotate)), _ptr(head_scale),
                                       _ptr(out), _stream()), "pq_rotate_quant_heads")
    return out


def pq_rotate_quant_groups(x, n_heads: int, rotate: bool, group: int = 128, clip: float = 1.0, out=None, scales=None):
    """x fp16 [T, n_heads*head_dim] -> (packed codes uint8 [T, C/2], group steps fp32 [T, C/group])."""
    _dev(x, torch.float16, "x")
    T, C = x.shape
    if C % n_heads:
        raise ValueError("shape mismatch")
    if out is None:
        out = torch.empty((T, C // 2), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((T, C // group), dtype=torch.float32, device=x.device)
    _check(lib().pq_rotate_quant_groups(_ptr(x), T, int(n_heads), C // n_heads, int(bool(rotate)), int(group),
                                        float(clip), _ptr(out), _ptr(scales), _stream()), "pq_rotate_quant_groups")
    return out, scales


def pq_rotate_f16(x, had_block: int, out=None):
    """x fp16 [M,K] -> its block-Hadamard rotation, fp16 [M,K]."""
    _dev(x, torch.float16, "x")
    if out is None:
        out = torch.empty_like(x)
    _check(lib().pq_rotate_f16(_ptr(x), x.shape[0], x.shape[1], int(had_block), _ptr(out), _stream()), "pq_rotate_f16")
    return out


def pq_silu_mul_rotate_quant(gate, up, had_block: int, act_scale: float, out=None):
    """gate, up fp16 [M,K] -> packed codes uint8 [M,K/2] of rotate(silu(gate) * up)."""
    _dev(gate, torch.float16, "gate")
    _dev(up, torch.float16, "up")
    if gate.shape != up.shape:
        raise ValueError("shape mismatch")
    M, K = gate.shape
    if out is None:
        out = torch.empty((M, K // 2), dtype=torch.uint8, device=gate.device)
    _check(lib().pq_silu_mul_rotate_quant(_ptr(gate), _ptr(up), M, K, int(had_block), float(act_scale), _ptr(out),
                                          _stream()), "pq_silu_mul_rotate_quant")
    return out


def pq_rmsnorm_quant(x, eps: float, act_scale: float, out=None):
    """x fp16 [M,K] -> packed codes uint8 [M,K/2] of x / rms(x)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if out is None:
        out = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    _check(lib().pq_rmsnorm_quant(_ptr(x), M, K, float(eps), float(act_scale), _ptr(out), _stream()),
           "pq_rmsnorm_quant")
    return out


def pq_rotate_quant_zp(x, had_block: int, act_scale: float, zero_point: int, out=None):
    """x fp16 [M,K] -> packed codes uint8 [M,K/2] of the quantizer with a zero-point (stored code = X_INT - 8)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if out is None:
        out = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    _check(lib().pq_rotate_quant_zp(_ptr(x), M, K, int(had_block), float(act_scale), int(zero_point), _ptr(out),
                                    _stream()), "pq_rotate_quant_zp")
    return out


def pq_zero_point_correction(wq, zero_point: int, out=None):
    """packed weights [N,K/2] -> int32 [N]: (8 - zero_point) * sum_k wq[n,k]."""
    _dev(wq, torch.uint8, "wq")
    N, K = wq.shape[0], wq.shape[1] * 2
    if out is None:
        out = torch.empty((N,), dtype=torch.int32, device=wq.device)
    _check(lib().pq_zero_point_correction(_ptr(wq), N, K, int(zero_point), _ptr(out), _stream()),
           "pq_zero_point_correction")
    return out


def pq_w4a4_gemm_zp(xq, wq, w_scale, act_scale, zp_corr, want_out=True, want_acc=False, out=None, acc=None,
                    workspace=None):
    """(acc + zp_corr[n]) * act_scale * w_scale[n] -> (out fp16 | None, raw acc int32 | None).
    With `workspace` (uint8 scratch) the call is pq_w4a4_gemm_zp_ws."""
    _dev(xq, torch.uint8, "xq")
    _dev(wq, torch.uint8, "wq")
    _dev(w_scale, torch.float32, "w_scale")
    _dev(zp_corr, torch.int32, "zp_corr")
    M, K = xq.shape[0], xq.shape[1] * 2
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or w_scale.numel() != N or zp_corr.numel() != N:
        raise ValueError("shape mismatch")
    if want_out and out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    if workspace is None:
        _check(lib().pq_w4a4_gemm_zp(_ptr(xq), _ptr(wq), _ptr(w_scale), float(act_scale), _ptr(zp_corr), M, N, K,
                                     _ptr(out), _ptr(acc), _stream()), "pq_w4a4_gemm_zp")
    else:
        _check(lib().pq_w4a4_gemm_zp_ws(_ptr(xq), _ptr(wq), _ptr(w_scale), float(act_scale), _ptr(zp_corr), M, N, K,
                                        _ptr(out), _ptr(acc), *_ws_args(workspace), _stream()), "pq_w4a4_gemm_zp_ws")
    return out, acc


def pq_w4a4_gemm_zp_ws(xq, wq, w_scale, act_scale, zp_corr, workspace, **kw):
    return pq_w4a4_gemm_zp(xq, wq, w_scale, act_scale, zp_corr, workspace=workspace, **kw)


def pq_calibrate_workspace_bytes(T: int, n_grid: int) -> int:
    return int(lib().pq_calibrate_workspace_bytes(T, int(n_grid)))


def pq_calibrate_static(x_cal, had_block: int, bits: int = 4, n_grid: int = 50, gamma_min: float = 0.5):
    """MSE grid search for the static step on the device.  Returns a device tensor fp32 [3 + n_grid]:
    best step, max-min step, best gamma, then the squared error of every candidate."""
    _dev(x_cal, torch.float16, "x_cal")
    T, K = x_cal.shape
    need = pq_calibrate_workspace_bytes(T, n_grid)
    ws = torch.empty((max(need, 256),), dtype=torch.uint8, device=x_cal.device)
    res = torch.empty((3 + n_grid,), dtype=torch.float32, device=x_cal.device)
    _check(lib().pq_calibrate_static(_ptr(x_cal), T, K, int(had_block), int(bits), int(n_grid), float(gamma_min),
                                     _ptr(res), _ptr(ws), ws.numel(), _stream()), "pq_calibrate_static")
    return res


def pq_calibrate_zp_workspace_bytes(T: int, n_candidates: int) -> int:
    return int(lib().pq_calibrate_zp_workspace_bytes(T, int(n_candidates)))


def pq_calibrate_static_zp(x_cal, had_block: int, n_gamma: int = 8, n_beta: int = 8, gamma_min: float = 0.5,
                           beta_min: float = 0.5):
    """MSE grid search over Eq. 1's (s, z) on the device.  Returns fp32 [6 + n_gamma * n_beta]: best s, best z,
    max-min s and z, arg-min (i, j), then the squared error of every candidate (index i * n_beta + j)."""
    _dev(x_cal, torch.float16, "x_cal")
    T, K = x_cal.shape
    n = n_gamma * n_beta
    ws = torch.empty((max(pq_calibrate_zp_workspace_bytes(T, n), 256),), dtype=torch.uint8, device=x_cal.device)
    res = torch.empty((6 + n,), dtype=torch.float32, device=x_cal.device)
    _check(lib().pq_calibrate_static_zp(_ptr(x_cal), T, K, int(had_block), int(n_gamma), int(n_beta), float(gamma_min),
                                        float(beta_min), _ptr(res), _ptr(ws), ws.numel(), _stream()),
           "pq_calibrate_static_zp")
    return res


def pq_set_gemm_variant(variant: int) -> int:
    return int(lib().pq_set_gemm_variant(int(variant)))


def pq_set_gemm_tile(tile: int) -> int:
    return int(lib().pq_set_gemm_tile(int(tile)))


def pq_set_gemm_f6_tile(tile: int) -> int:
    return int(lib().pq_set_gemm_f6_tile(int(tile)))


def pq_probe_mfma_i8(operands: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor) -> float:
    """Launches the matrix-pipe probe; returns the integer operations of the launch."""
    _check(lib().pq_probe_mfma_i8(_ptr(operands), operands.numel() * operands.element_size(), int(iters), int(workgroups),
                                  _ptr(sink), _stream()), "pq_probe_mfma_i8")
    return float(workgroups) * 4 * iters * 16 * 65536


def pq_f6_tiles_bytes(rows: int, K: int) -> int:
    return int(lib().pq_f6_tiles_bytes(rows, K))


def pq_repack_f6(codes: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """packed codes uint8 [rows,K/2] -> register images of the 6-bit matrix instruction (uint8, flat)."""
    _dev(codes, torch.uint8, "codes")
    rows, K = codes.shape[0], codes.shape[1] * 2
    if out is None:
        out = torch.empty((max(pq_f6_tiles_bytes(rows, K), 16),), dtype=torch.uint8, device=codes.device)
    _check(lib().pq_repack_f6(_ptr(codes), rows, K, _ptr(out), _stream()), "pq_repack_f6")
    return out


def pq_w4a4_gemm_f6(x_tiles, w_tiles, w_scale, act_scale, M: int, N: int, K: int, want_out=True, want_acc=False,
                    out=None, acc=None):
    """tiles of [M,K] x tiles of [N,K] -> (out fp16 [M,N] | None, acc int32 [M,N] | None)."""
    _dev(x_tiles, torch.uint8, "x_tiles")
    _dev(w_tiles, torch.uint8, "w_tiles")
    _dev(w_scale, torch.float32, "w_scale")
    if (M > 0 and x_tiles.numel() < pq_f6_tiles_bytes(M, K)) or w_tiles.numel() < pq_f6_tiles_bytes(N, K) or w_scale.numel() != N:
        raise ValueError("shape mismatch")
    if want_out and out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x_tiles.device)
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=x_tiles.device)
    _check(lib().pq_w4a4_gemm_f6(_ptr(x_tiles), _ptr(w_tiles), _ptr(w_scale), float(act_scale), M, N, K, _ptr(out),
                                 _ptr(acc), _stream()), "pq_w4a4_gemm_f6")
    return out, acc


def pq_linear_f6_workspace_bytes(M: int, K: int, had_block: int = 1) -> int:
    return int(lib().pq_linear_f6_workspace_bytes(M, K, int(had_block)))


def pq_rotate_quant_f6(x, had_block: int, act_scale: float, out=None, codes=None):
    """x fp16 [M,K] -> the f6 tiles of its codes (uint8, pq_f6_tiles_bytes(M,K)); codes: optional uint8 [M,K/2]
    that receives the canonical packed codes as well."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if out is None:
        out = torch.empty((pq_f6_tiles_bytes(M, K),), dtype=torch.uint8, device=x.device)
    if codes is not None:
        _dev(codes, torch.uint8, "codes")
    _check(lib().pq_rotate_quant_f6(_ptr(x), M, K, int(had_block), float(act_scale), _ptr(out), _ptr(codes), _stream()),
           "pq_rotate_quant_f6")
    return out


def pq_linear_f6(x, w_tiles, w_scale, act_scale, had_block, out=None, workspace=None):
    """The whole layer with prepacked weights (pq_repack_f6).  Returns (out fp16 [M,N], workspace uint8: the
    activation tiles, and behind them the canonical packed codes if had_block > 512)."""
    _dev(x, torch.float16, "x")
    _dev(w_tiles, torch.uint8, "w_tiles")
    _dev(w_scale, torch.float32, "w_scale")
    M, K = x.shape
    N = w_scale.numel()
    if w_tiles.numel() < pq_f6_tiles_bytes(N, K):
        raise ValueError("shape mismatch")
    need = pq_linear_f6_workspace_bytes(M, K, had_block)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().pq_linear_f6(_ptr(x), _ptr(w_tiles), _ptr(w_scale), float(act_scale), int(had_block), M, N, K, _ptr(out),
                              _ptr(workspace), workspace.numel(), _stream()), "pq_linear_f6")
    return out, workspace


def pq_probe_mfma_f6(operands: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor) -> float:
    """Launches the 6-bit matrix-instruction probe; returns the operations of the launch."""
    _check(lib().pq_probe_mfma_f6(_ptr(operands), operands.numel() * operands.element_size(), int(iters), int(workgroups),
                                  _ptr(sink), _stream()), "pq_probe_mfma_f6")
    return float(workgroups) * 4 * iters * 16 * 131072


def pq_probe_f6_product(a_codes: torch.Tensor, b_codes: torch.Tensor) -> torch.Tensor:
    """int8 codes [32,K] x [32,K] -> int32 [32,32] through the 6-bit floating-point matrix instruction."""
    _dev(a_codes, torch.int8, "a_codes")
    _dev(b_codes, torch.int8, "b_codes")
    if a_codes.shape != b_codes.shape or a_codes.shape[0] != 32:
        raise ValueError("shape mismatch")
    out = torch.empty((32, 32), dtype=torch.int32, device=a_codes.device)
    _check(lib().pq_probe_f6_product(_ptr(a_codes), _ptr(b_codes), a_codes.shape[1], _ptr(out), _stream()),
           "pq_probe_f6_product")
    return out


def pq_probe_stream_read(src: torch.Tensor, sink: torch.Tensor) -> int:
    """Launches the read-only probe over the whole tensor; returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    _check(lib().pq_probe_stream_read(_ptr(src), nbytes, _ptr(sink), _stream()), "pq_probe_stream_read")
    return nbytes
