"""Thin ctypes binding over libsvdq.so: argument marshalling only.

Every step of the layer runs inside the library (host-side offline quantization in C++,
run-time kernels in HIP); PyTorch is used here only to own device memory and streams.
Function names mirror the C ABI declared in ``include/svdq.h``.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsvdq.so")

OPT_SKIP_LOWRANK = 1
OPT_UNFUSED = 2
OPT_KSPLIT_SHIFT = 8
OPT_ACT_CHUNK_SHIFT = 12

EXPORTS = [
    "svdq_status_string", "svdq_last_hip_error", "svdq_prepared_sizes", "svdq_prepare", "svdq_pack",
    "svdq_unpack_wcodes", "svdq_unpack_wscales", "svdq_unpack_l1s", "svdq_unpack_l2", "svdq_append_lora", "svdq_prepare_refined", "svdq_prepare_gptq",
    "svdq_fp4_prepared_sizes", "svdq_fp4_prepare", "svdq_fp4_pack", "svdq_fp4_unpack_wcodes", "svdq_fp4_unpack_wscales",
    "svdq_fp4_workspace_bytes", "svdq_fp4_linear_forward", "svdq_fp4_debug_act",
    "svdq_w8a8_prepared_sizes", "svdq_w8a8_prepare", "svdq_w8a8_pack", "svdq_w8a8_unpack_wcodes", "svdq_w8a8_unpack_wscales",
    "svdq_w8a8_workspace_bytes", "svdq_w8a8_linear_forward", "svdq_w8a8_debug_act", "svdq_w4a16_forward", "svdq_w4a16_workspace_bytes",
    "svdq_workspace_bytes", "svdq_linear_forward", "svdq_debug_act", "svdq_debug_group_acc",
    "svdq_forward_options", "svdq_profile_event", "svdq_mfma_peak_probe", "svdq_linear_forward_static",
    "svdq_debug_launch_plan",
]


class SvdqError(RuntimeError):
    pass


class Shape(C.Structure):
    _fields_ = [("K", C.c_int), ("N", C.c_int), ("rank", C.c_int), ("group", C.c_int), ("alpha", C.c_float)]


class Sizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("rinv", "l1s", "l2", "wcodes", "wscales", "bias")]


class LayerDev(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("rinv", "l1s", "l2", "wcodes", "wscales", "bias")] + [("shape", Shape)]


_lib = None


def lib() -> C.CDLL:
    """Load libsvdq.so (built in-tree by ``build.py``); raise loudly if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SvdqError(
                f"{LIB_PATH} not found: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
                "There is no CPU fallback for the layer.")
        L = C.CDLL(LIB_PATH)
        L.svdq_status_string.restype = C.c_char_p
        L.svdq_status_string.argtypes = [C.c_int]
        L.svdq_workspace_bytes.restype = C.c_size_t
        L.svdq_workspace_bytes.argtypes = [C.c_int, C.POINTER(Shape)]
        L.svdq_debug_launch_plan.argtypes = [C.POINTER(Shape), C.c_int, C.POINTER(C.c_int32)]
        L.svdq_prepared_sizes.argtypes = [C.POINTER(Shape), C.POINTER(Sizes)]
        vp = C.c_void_p
        L.svdq_prepare.argtypes = [C.POINTER(Shape)] + [vp] * 9
        L.svdq_pack.argtypes = [C.POINTER(Shape)] + [vp] * 12
        for n in ("svdq_unpack_wcodes", "svdq_unpack_wscales", "svdq_unpack_l1s", "svdq_unpack_l2"):
            getattr(L, n).argtypes = [C.POINTER(Shape), vp, vp]
        L.svdq_append_lora.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, C.c_int, C.c_float, C.POINTER(Shape), vp, vp]
        L.svdq_prepare_refined.argtypes = [C.POINTER(Shape), vp, vp, vp, C.c_int] + [vp] * 8
        L.svdq_prepare_gptq.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, C.c_int, C.c_float] + [vp] * 7
        L.svdq_fp4_workspace_bytes.restype = C.c_size_t
        L.svdq_fp4_workspace_bytes.argtypes = [C.c_int, C.POINTER(Shape)]
        L.svdq_fp4_prepared_sizes.argtypes = [C.POINTER(Shape), C.POINTER(Sizes)]
        L.svdq_fp4_prepare.argtypes = [C.POINTER(Shape)] + [vp] * 9
        L.svdq_fp4_pack.argtypes = [C.POINTER(Shape)] + [vp] * 12
        for n in ("svdq_fp4_unpack_wcodes", "svdq_fp4_unpack_wscales"):
            getattr(L, n).argtypes = [C.POINTER(Shape), vp, vp]
        L.svdq_fp4_linear_forward.argtypes = [C.POINTER(LayerDev), vp, C.c_int, vp, vp, C.c_size_t, vp]
        L.svdq_fp4_debug_act.argtypes = [C.POINTER(LayerDev), vp, C.c_int, vp, vp, vp, vp]
        L.svdq_w4a16_forward.argtypes = [C.POINTER(LayerDev), vp, C.c_int, vp, vp, C.c_size_t, vp]
        L.svdq_w4a16_workspace_bytes.argtypes = [C.c_int, C.POINTER(Shape)]
        L.svdq_w4a16_workspace_bytes.restype = C.c_size_t
        L.svdq_w8a8_workspace_bytes.restype = C.c_size_t
        L.svdq_w8a8_workspace_bytes.argtypes = [C.c_int, C.POINTER(Shape)]
        L.svdq_w8a8_prepared_sizes.argtypes = [C.POINTER(Shape), C.POINTER(Sizes)]
        L.svdq_w8a8_prepare.argtypes = [C.POINTER(Shape)] + [vp] * 9
        L.svdq_w8a8_pack.argtypes = [C.POINTER(Shape)] + [vp] * 12
        for n in ("svdq_w8a8_unpack_wcodes", "svdq_w8a8_unpack_wscales"):
            getattr(L, n).argtypes = [C.POINTER(Shape), vp, vp]
        L.svdq_w8a8_linear_forward.argtypes = [C.POINTER(LayerDev), vp, C.c_int, vp, vp, C.c_size_t, vp]
        L.svdq_w8a8_debug_act.argtypes = [C.POINTER(LayerDev), vp, C.c_int, vp, vp, vp, vp]
        L.svdq_linear_forward.argtypes = [C.POINTER(LayerDev), vp, C.c_int, vp, vp, C.c_size_t, vp]
        L.svdq_linear_forward_static.argtypes = [C.POINTER(LayerDev), vp, C.c_int, vp, vp]
        L.svdq_debug_act.argtypes = [C.POINTER(LayerDev), vp, C.c_int, vp, vp, vp, vp]
        L.svdq_debug_group_acc.argtypes = [C.POINTER(LayerDev), vp, C.c_int] + [C.c_int] * 4 + [vp, vp]
        L.svdq_forward_options.argtypes = [C.c_int]
        L.svdq_profile_event.argtypes = [vp]
        L.svdq_mfma_peak_probe.argtypes = [C.c_int, C.c_int, vp, C.c_size_t, vp, C.POINTER(C.c_double)]
        _lib = L
    return _lib


def _check(status: int, what: str) -> None:
    if status != 0:
        L = lib()
        msg = L.svdq_status_string(status).decode()
        extra = f" (hipError {L.svdq_last_hip_error()})" if status == -5 else ""
        raise SvdqError(f"{what}: {msg}{extra}")


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def make_shape(K: int, N: int, rank: int, alpha: float = 0.5, group: int = 64) -> Shape:
    return Shape(K, N, rank, group, alpha)


@dataclass
class PreparedHost:
    """Native (kernel-ordered) host buffers of one quantized layer."""
    shape: Shape
    rinv: np.ndarray
    l1s: np.ndarray
    l2: np.ndarray
    wcodes: np.ndarray
    wscales: np.ndarray
    bias: np.ndarray


def _is_fp4(shape: Shape) -> bool:
    return shape.group == 32


def _is_w8(shape: Shape) -> bool:
    return shape.group == 0


def _alloc_prepared(shape: Shape) -> PreparedHost:
    sz = Sizes()
    if _is_fp4(shape):
        _check(lib().svdq_fp4_prepared_sizes(C.byref(shape), C.byref(sz)), "svdq_fp4_prepared_sizes")
    elif _is_w8(shape):
        _check(lib().svdq_w8a8_prepared_sizes(C.byref(shape), C.byref(sz)), "svdq_w8a8_prepared_sizes")
    else:
        _check(lib().svdq_prepared_sizes(C.byref(shape), C.byref(sz)), "svdq_prepared_sizes")
    return PreparedHost(
        shape=shape,
        rinv=np.zeros(sz.rinv // 4, np.float32),
        l1s=np.zeros(sz.l1s // 2, np.uint16),
        l2=np.zeros(sz.l2 // 2, np.uint16),
        wcodes=np.zeros(sz.wcodes, np.uint8),
        wscales=np.zeros(sz.wscales, np.uint8) if _is_fp4(shape) else np.zeros(sz.wscales // 2, np.uint16),
        bias=np.zeros(sz.bias // 4, np.float32),
    )


def svdq_prepare(W: np.ndarray, x_absmax: np.ndarray, rank: int, alpha: float = 0.5,
                 bias: Optional[np.ndarray] = None) -> PreparedHost:
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    x_absmax = np.ascontiguousarray(x_absmax, dtype=np.float32)
    assert x_absmax.shape == (K,)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    shape = make_shape(K, N, rank, alpha)
    out = _alloc_prepared(shape)
    _check(lib().svdq_prepare(C.byref(shape), _ptr(W), _ptr(x_absmax), _ptr(b), _ptr(out.rinv), _ptr(out.l1s),
                              _ptr(out.l2), _ptr(out.wcodes), _ptr(out.wscales), _ptr(out.bias)), "svdq_prepare")
    return out


def svdq_pack(rinv, l1s_bits, l2_bits, qw, sw_f16, bias=None, alpha: float = 0.5) -> PreparedHost:
    """Pack canonical arrays (e.g. from another quantizer) into native buffers."""
    qw = np.ascontiguousarray(qw, dtype=np.int8)
    K, N = qw.shape
    l1s_bits = np.ascontiguousarray(l1s_bits, dtype=np.uint16)
    rank = l1s_bits.shape[1] if l1s_bits.ndim == 2 else 0
    l2_bits = np.ascontiguousarray(l2_bits, dtype=np.uint16)
    sw = np.ascontiguousarray(np.asarray(sw_f16).view(np.uint16))
    rinv = np.ascontiguousarray(rinv, dtype=np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    shape = make_shape(K, N, rank, alpha)
    out = _alloc_prepared(shape)
    _check(lib().svdq_pack(C.byref(shape), _ptr(rinv), _ptr(l1s_bits) if rank else None, _ptr(l2_bits) if rank else None,
                           _ptr(qw), _ptr(sw), _ptr(b), _ptr(out.rinv), _ptr(out.l1s), _ptr(out.l2),
                           _ptr(out.wcodes), _ptr(out.wscales), _ptr(out.bias)), "svdq_pack")
    return out


def svdq_unpack(p: PreparedHost):
    """Canonical views of a prepared layer: dict(rinv, l1s bf16 [K,r], l2 bf16 [r,N], qw int8 [K,N], sw fp16 [G,N], bias)."""
    K, N, r = p.shape.K, p.shape.N, p.shape.rank
    G = K // 64
    qw = np.zeros((K, N), np.int8)
    sw = np.zeros((G, N), np.uint16)
    l1s = np.zeros((K, r), np.uint16)
    l2 = np.zeros((r, N), np.uint16)
    L = lib()
    _check(L.svdq_unpack_wcodes(C.byref(p.shape), _ptr(p.wcodes), _ptr(qw)), "svdq_unpack_wcodes")
    _check(L.svdq_unpack_wscales(C.byref(p.shape), _ptr(p.wscales), _ptr(sw)), "svdq_unpack_wscales")
    if r > 0:
        _check(L.svdq_unpack_l1s(C.byref(p.shape), _ptr(p.l1s), _ptr(l1s)), "svdq_unpack_l1s")
        _check(L.svdq_unpack_l2(C.byref(p.shape), _ptr(p.l2), _ptr(l2)), "svdq_unpack_l2")
    return {"rinv": p.rinv.copy(), "l1s": l1s, "l2": l2, "qw": qw, "sw": sw.view(np.float16), "bias": p.bias[:N].copy()}


def svdq_prepare_refined(W: np.ndarray, x_absmax: np.ndarray, rank: int, iterations: int, alpha: float = 0.5,
                         bias: Optional[np.ndarray] = None, fp4: bool = False):
    """Prepare with the iterative update of the low-rank branch.  Returns (PreparedHost, errors of all iterates, picked index)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    x_absmax = np.ascontiguousarray(x_absmax, dtype=np.float32)
    assert x_absmax.shape == (K,)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    shape = make_shape(K, N, rank, alpha, group=32 if fp4 else 64)
    out = _alloc_prepared(shape)
    errors = np.zeros(iterations + 1, np.float64)
    pick = C.c_int(-1)
    _check(lib().svdq_prepare_refined(C.byref(shape), _ptr(W), _ptr(x_absmax), _ptr(b), int(iterations), _ptr(out.rinv),
                                      _ptr(out.l1s), _ptr(out.l2), _ptr(out.wcodes), _ptr(out.wscales), _ptr(out.bias),
                                      _ptr(errors), C.byref(pick)), "svdq_prepare_refined")
    return out, errors, pick.value


def svdq_prepare_gptq(W: np.ndarray, x_absmax: np.ndarray, rank: int, x_cal: np.ndarray, damp: float = 0.01,
                      alpha: float = 0.5, bias: Optional[np.ndarray] = None, fp4: bool = False):
    """Prepare an INT4 (or MXFP4) layer with the residual quantized by GPTQ on calibration activations x_cal fp32 [Mc, K].
    Returns (PreparedHost, (objective of round-to-nearest, objective of the packed codes))."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    x_absmax = np.ascontiguousarray(x_absmax, dtype=np.float32)
    x_cal = np.ascontiguousarray(x_cal, dtype=np.float32)
    assert x_absmax.shape == (K,) and x_cal.ndim == 2 and x_cal.shape[1] == K
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    shape = make_shape(K, N, rank, alpha, group=32 if fp4 else 64)
    out = _alloc_prepared(shape)
    objective = np.zeros(2, np.float64)
    _check(lib().svdq_prepare_gptq(C.byref(shape), _ptr(W), _ptr(x_absmax), _ptr(b), _ptr(x_cal), int(x_cal.shape[0]),
                                   float(damp), _ptr(out.rinv), _ptr(out.l1s), _ptr(out.l2), _ptr(out.wcodes),
                                   _ptr(out.wscales), _ptr(out.bias), _ptr(objective)), "svdq_prepare_gptq")
    return out, (float(objective[0]), float(objective[1]))


def svdq_fp4_prepare(W: np.ndarray, x_absmax: np.ndarray, rank: int, alpha: float = 0.5,
                     bias: Optional[np.ndarray] = None) -> PreparedHost:
    """The MXFP4 variant of svdq_prepare (shape.group = 32)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    x_absmax = np.ascontiguousarray(x_absmax, dtype=np.float32)
    assert x_absmax.shape == (K,)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    shape = make_shape(K, N, rank, alpha, group=32)
    out = _alloc_prepared(shape)
    _check(lib().svdq_fp4_prepare(C.byref(shape), _ptr(W), _ptr(x_absmax), _ptr(b), _ptr(out.rinv), _ptr(out.l1s),
                                  _ptr(out.l2), _ptr(out.wcodes), _ptr(out.wscales), _ptr(out.bias)), "svdq_fp4_prepare")
    return out


def svdq_fp4_pack(rinv, l1s_bits, l2_bits, qw, bw, bias=None, alpha: float = 0.5) -> PreparedHost:
    """Pack canonical MXFP4 arrays: qw uint8 [K, N] codes 0..15, bw uint8 [K/32, N] scale bytes."""
    qw = np.ascontiguousarray(qw, dtype=np.uint8)
    bw = np.ascontiguousarray(bw, dtype=np.uint8)
    K, N = qw.shape
    assert bw.shape == (K // 32, N)
    l1s_bits = np.ascontiguousarray(l1s_bits, dtype=np.uint16)
    rank = l1s_bits.shape[1] if l1s_bits.ndim == 2 else 0
    l2_bits = np.ascontiguousarray(l2_bits, dtype=np.uint16)
    rinv = np.ascontiguousarray(rinv, dtype=np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    shape = make_shape(K, N, rank, alpha, group=32)
    out = _alloc_prepared(shape)
    _check(lib().svdq_fp4_pack(C.byref(shape), _ptr(rinv), _ptr(l1s_bits) if rank else None, _ptr(l2_bits) if rank else None,
                               _ptr(qw), _ptr(bw), _ptr(b), _ptr(out.rinv), _ptr(out.l1s), _ptr(out.l2),
                               _ptr(out.wcodes), _ptr(out.wscales), _ptr(out.bias)), "svdq_fp4_pack")
    return out


def svdq_fp4_unpack(p: PreparedHost):
    """Canonical views of an MXFP4 layer: dict(rinv, l1s, l2, qw uint8 [K,N], bw uint8 [K/32,N], bias)."""
    K, N, r = p.shape.K, p.shape.N, p.shape.rank
    qw = np.zeros((K, N), np.uint8)
    bw = np.zeros((K // 32, N), np.uint8)
    l1s = np.zeros((K, r), np.uint16)
    l2 = np.zeros((r, N), np.uint16)
    L = lib()
    _check(L.svdq_fp4_unpack_wcodes(C.byref(p.shape), _ptr(p.wcodes), _ptr(qw)), "svdq_fp4_unpack_wcodes")
    _check(L.svdq_fp4_unpack_wscales(C.byref(p.shape), _ptr(p.wscales), _ptr(bw)), "svdq_fp4_unpack_wscales")
    if r > 0:
        _check(L.svdq_unpack_l1s(C.byref(p.shape), _ptr(p.l1s), _ptr(l1s)), "svdq_unpack_l1s")
        _check(L.svdq_unpack_l2(C.byref(p.shape), _ptr(p.l2), _ptr(l2)), "svdq_unpack_l2")
    return {"rinv": p.rinv.copy(), "l1s": l1s, "l2": l2, "qw": qw, "bw": bw, "bias": p.bias[:N].copy()}


def svdq_w8a8_prepare(W: np.ndarray, x_absmax: np.ndarray, rank: int = 16, alpha: float = 0.5,
                      bias: Optional[np.ndarray] = None) -> PreparedHost:
    """The 8-bit setting (shape.group = 0): per-channel INT8 residual, rank-r 16-bit branch."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    x_absmax = np.ascontiguousarray(x_absmax, dtype=np.float32)
    assert x_absmax.shape == (K,)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    shape = make_shape(K, N, rank, alpha, group=0)
    out = _alloc_prepared(shape)
    _check(lib().svdq_w8a8_prepare(C.byref(shape), _ptr(W), _ptr(x_absmax), _ptr(b), _ptr(out.rinv), _ptr(out.l1s),
                                   _ptr(out.l2), _ptr(out.wcodes), _ptr(out.wscales), _ptr(out.bias)), "svdq_w8a8_prepare")
    return out


def svdq_w8a8_pack(rinv, l1s_bits, l2_bits, qw, sw_f16, bias=None, alpha: float = 0.5) -> PreparedHost:
    """Pack canonical W8A8 arrays: qw int8 [K, N], sw fp16 [N]."""
    qw = np.ascontiguousarray(qw, dtype=np.int8)
    K, N = qw.shape
    sw = np.ascontiguousarray(np.asarray(sw_f16).view(np.uint16))
    assert sw.shape == (N,)
    l1s_bits = np.ascontiguousarray(l1s_bits, dtype=np.uint16)
    rank = l1s_bits.shape[1] if l1s_bits.ndim == 2 else 0
    l2_bits = np.ascontiguousarray(l2_bits, dtype=np.uint16)
    rinv = np.ascontiguousarray(rinv, dtype=np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    shape = make_shape(K, N, rank, alpha, group=0)
    out = _alloc_prepared(shape)
    _check(lib().svdq_w8a8_pack(C.byref(shape), _ptr(rinv), _ptr(l1s_bits) if rank else None, _ptr(l2_bits) if rank else None,
                                _ptr(qw), _ptr(sw), _ptr(b), _ptr(out.rinv), _ptr(out.l1s), _ptr(out.l2),
                                _ptr(out.wcodes), _ptr(out.wscales), _ptr(out.bias)), "svdq_w8a8_pack")
    return out


def svdq_w8a8_unpack(p: PreparedHost):
    """Canonical views of a W8A8 layer: dict(rinv, l1s, l2, qw int8 [K,N], sw fp16 [N], bias)."""
    K, N, r = p.shape.K, p.shape.N, p.shape.rank
    qw = np.zeros((K, N), np.int8)
    sw = np.zeros(N, np.uint16)
    l1s = np.zeros((K, r), np.uint16)
    l2 = np.zeros((r, N), np.uint16)
    L = lib()
    _check(L.svdq_w8a8_unpack_wcodes(C.byref(p.shape), _ptr(p.wcodes), _ptr(qw)), "svdq_w8a8_unpack_wcodes")
    _check(L.svdq_w8a8_unpack_wscales(C.byref(p.shape), _ptr(p.wscales), _ptr(sw)), "svdq_w8a8_unpack_wscales")
    if r > 0:
        _check(L.svdq_unpack_l1s(C.byref(p.shape), _ptr(p.l1s), _ptr(l1s)), "svdq_unpack_l1s")
        _check(L.svdq_unpack_l2(C.byref(p.shape), _ptr(p.l2), _ptr(l2)), "svdq_unpack_l2")
    return {"rinv": p.rinv.copy(), "l1s": l1s, "l2": l2, "qw": qw, "sw": sw.view(np.float16), "bias": p.bias[:N].copy()}


def svdq_append_lora(p: PreparedHost, down: np.ndarray, up: np.ndarray, scale: float = 1.0) -> PreparedHost:
    """A layer with the adapter `scale * down @ up` appended to its 16-bit branch; everything else is shared with `p`."""
    down = np.ascontiguousarray(down, dtype=np.float32)
    up = np.ascontiguousarray(up, dtype=np.float32)
    r_add = down.shape[1]
    assert down.shape == (p.shape.K, r_add) and up.shape == (r_add, p.shape.N)
    has = p.shape.rank > 0
    want = make_shape(p.shape.K, p.shape.N, (p.shape.rank + r_add + 15) // 16 * 16, p.shape.alpha, p.shape.group)
    blank = _alloc_prepared(want)
    l1s, l2 = blank.l1s, blank.l2
    ns = Shape()
    _check(lib().svdq_append_lora(C.byref(p.shape), _ptr(p.l1s) if has else None, _ptr(p.l2) if has else None, _ptr(down),
                                  _ptr(up), r_add, float(scale), C.byref(ns), _ptr(l1s), _ptr(l2)), "svdq_append_lora")
    assert ns.rank == want.rank
    return PreparedHost(shape=ns, rinv=p.rinv, l1s=l1s, l2=l2, wcodes=p.wcodes, wscales=p.wscales, bias=p.bias)


def svdq_forward_options(flags: int) -> int:
    return lib().svdq_forward_options(int(flags))


def svdq_mfma_peak_probe(kind: int, iters: int, sink, stream) -> float:
    """Enqueue the register-only MFMA loop (kind 0: int8, 1: 6-bit operands) on `stream`; returns the operations of one launch."""
    ops = C.c_double()
    _check(lib().svdq_mfma_peak_probe(int(kind), int(iters), sink.data_ptr(), sink.numel() * sink.element_size(),
                                      stream.cuda_stream, C.byref(ops)), "svdq_mfma_peak_probe")
    return float(ops.value)


def svdq_profile_event(event_handle: Optional[int]) -> None:
    _check(lib().svdq_profile_event(event_handle), "svdq_profile_event")


PLAN_FIELDS = ("act_runs", "act_groups_per_run", "act_waves", "act_leading_slices", "act_leading_runs", "act_leading_groups_per_run",
               "act_workgroups", "act_lds_bytes", "gemm_tiles", "gemm_split_tiles", "gemm_ksplit", "gemm_workgroups",
               "parked_bytes_256", "parked_h_bytes_256", "arrival_words", "workspace_bytes_256")


def svdq_debug_launch_plan(M: int, shape: Shape) -> dict:
    """The launch plan of a forward of M tokens (host only): see include/svdq.h."""
    out = (C.c_int32 * 16)()
    _check(lib().svdq_debug_launch_plan(C.byref(shape), int(M), out), "svdq_debug_launch_plan")
    return dict(zip(PLAN_FIELDS, (int(v) for v in out)))


def svdq_workspace_bytes(M: int, shape: Shape) -> int:
    if _is_fp4(shape):
        return int(lib().svdq_fp4_workspace_bytes(int(M), C.byref(shape)))
    if _is_w8(shape):
        return int(lib().svdq_w8a8_workspace_bytes(int(M), C.byref(shape)))
    return int(lib().svdq_workspace_bytes(int(M), C.byref(shape)))


class DeviceLayer:
    """A prepared layer resident in HBM (torch tensors own the memory) plus its forward call."""

    def __init__(self, prepared: PreparedHost, device: str = "cuda:0"):
        import torch

        if not torch.cuda.is_available():
            raise SvdqError("no GPU visible: the SVDQuant layer has no CPU path")
        self.torch = torch
        self.device = torch.device(device)
        self.shape = prepared.shape
        self.K, self.N, self.rank = prepared.shape.K, prepared.shape.N, prepared.shape.rank
        self.G = self.K // 64
        self.fp4 = _is_fp4(prepared.shape)
        self.w8 = _is_w8(prepared.shape)
        up = lambda a: torch.from_numpy(a.view(np.uint8) if a.dtype != np.uint8 else a).to(self.device)
        self._bufs = {n: up(getattr(prepared, n)) for n in ("rinv", "l1s", "l2", "wcodes", "wscales", "bias")}
        self.cdesc = LayerDev(*[self._bufs[n].data_ptr() for n in ("rinv", "l1s", "l2", "wcodes", "wscales", "bias")],
                              prepared.shape)

    def workspace(self, M: int):
        n = svdq_workspace_bytes(M, self.shape)
        if n == 0:
            raise SvdqError("unsupported shape")
        return self.torch.empty(n, dtype=self.torch.uint8, device=self.device)

    def forward(self, x, out=None, workspace=None, stream=None):
        """x: torch bf16 [M, K] on the GPU.  Returns bf16 [M, N].  Enqueues only; does not synchronise."""
        torch = self.torch
        assert x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape[1] == self.K and x.is_cuda
        M = x.shape[0]
        if out is None:
            out = torch.empty((M, self.N), dtype=torch.bfloat16, device=x.device)
        if workspace is None:
            workspace = self.workspace(M)
        s = torch.cuda.current_stream(x.device) if stream is None else stream
        name = "svdq_fp4_linear_forward" if self.fp4 else "svdq_w8a8_linear_forward" if self.w8 else "svdq_linear_forward"
        _check(getattr(lib(), name)(C.byref(self.cdesc), x.data_ptr(), M, out.data_ptr(), workspace.data_ptr(),
                                    workspace.numel(), s.cuda_stream), name)
        self._last_ws, self._last_M = workspace, M
        return out

    def forward_static(self, x, out, stream=None):
        """The INT4 forward on the library's own static workspace (no allocation inside the call); `out` is the caller's."""
        torch = self.torch
        assert not self.fp4 and not self.w8, "the static-workspace entry point exists for the INT4 layer"
        assert x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape[1] == self.K and x.is_cuda
        assert out.dtype == torch.bfloat16 and out.is_contiguous() and tuple(out.shape) == (x.shape[0], self.N)
        s = torch.cuda.current_stream(x.device) if stream is None else stream
        _check(lib().svdq_linear_forward_static(C.byref(self.cdesc), x.data_ptr(), x.shape[0], out.data_ptr(), s.cuda_stream),
               "svdq_linear_forward_static")
        return out

    def forward_w4a16(self, x, out=None, workspace=None, stream=None):
        """The INT4 layer applied to 16-bit activations (no activation quantization); small batches."""
        torch = self.torch
        assert not self.fp4 and not self.w8, "W4A16 uses a layer prepared for INT4 (group 64)"
        assert x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape[1] == self.K and x.is_cuda
        M = x.shape[0]
        if out is None:
            out = torch.empty((M, self.N), dtype=torch.bfloat16, device=x.device)
        if workspace is None:      # H and its bf16 parts only
            workspace = torch.empty(int(lib().svdq_w4a16_workspace_bytes(int(M), C.byref(self.shape))), dtype=torch.uint8, device=self.device)
        s = torch.cuda.current_stream(x.device) if stream is None else stream
        _check(lib().svdq_w4a16_forward(C.byref(self.cdesc), x.data_ptr(), M, out.data_ptr(), workspace.data_ptr(),
                                        workspace.numel(), s.cuda_stream), "svdq_w4a16_forward")
        return out

    def debug_act(self, workspace=None, M=None):
        """Canonical codes int8 [M,K], scales fp16 [M,G], H fp32 [M,r] of the last forward (numpy)."""
        torch = self.torch
        workspace = self._last_ws if workspace is None else workspace
        M = self._last_M if M is None else M
        H = torch.empty((M, max(self.rank, 1)), dtype=torch.float32, device=self.device)
        s = torch.cuda.current_stream(self.device)
        if self.fp4:      # codes uint8 [M,K] (0..15), scale bytes uint8 [M,K/32]
            codes = torch.empty((M, self.K), dtype=torch.uint8, device=self.device)
            bx = torch.empty((M, self.K // 32), dtype=torch.uint8, device=self.device)
            _check(lib().svdq_fp4_debug_act(C.byref(self.cdesc), workspace.data_ptr(), M, codes.data_ptr(), bx.data_ptr(),
                                            H.data_ptr() if self.rank else None, s.cuda_stream), "svdq_fp4_debug_act")
            torch.cuda.synchronize(self.device)
            return codes.cpu().numpy(), bx.cpu().numpy(), (H.cpu().numpy() if self.rank else None)
        codes = torch.empty((M, self.K), dtype=torch.int8, device=self.device)
        if self.w8:       # codes int8 [M,K], one fp16 scale per token
            sx = torch.empty((M,), dtype=torch.float16, device=self.device)
            _check(lib().svdq_w8a8_debug_act(C.byref(self.cdesc), workspace.data_ptr(), M, codes.data_ptr(), sx.data_ptr(),
                                             H.data_ptr() if self.rank else None, s.cuda_stream), "svdq_w8a8_debug_act")
            torch.cuda.synchronize(self.device)
            return codes.cpu().numpy(), sx.cpu().numpy(), (H.cpu().numpy() if self.rank else None)
        sx = torch.empty((M, self.G), dtype=torch.float16, device=self.device)
        _check(lib().svdq_debug_act(C.byref(self.cdesc), workspace.data_ptr(), M, codes.data_ptr(), sx.data_ptr(),
                                    H.data_ptr() if self.rank else None, s.cuda_stream), "svdq_debug_act")
        torch.cuda.synchronize(self.device)
        return codes.cpu().numpy(), sx.cpu().numpy(), (H.cpu().numpy() if self.rank else None)

    def debug_group_acc(self, m0, m1, n0, n1, workspace=None, M=None):
        """Exact int32 group sums of a window, int32 [m1-m0, n1-n0, G] (numpy)."""
        torch = self.torch
        workspace = self._last_ws if workspace is None else workspace
        M = self._last_M if M is None else M
        out = torch.zeros((m1 - m0, n1 - n0, self.G), dtype=torch.int32, device=self.device)
        s = torch.cuda.current_stream(self.device)
        _check(lib().svdq_debug_group_acc(C.byref(self.cdesc), workspace.data_ptr(), M, m0, m1, n0, n1, out.data_ptr(),
                                          s.cuda_stream), "svdq_debug_group_acc")
        torch.cuda.synchronize(self.device)
        return out.cpu().numpy()


def bf16_tensor_from_bits(bits: np.ndarray, device="cuda:0"):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on the device."""
    import torch

    return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)


def bits_from_bf16_tensor(t) -> np.ndarray:
    import torch

    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
