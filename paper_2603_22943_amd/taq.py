"""Thin ctypes binding of libtaq.so: same names as the C ABI in include/taq.h.

Argument marshalling only: torch tensors supply device memory and the current
HIP stream; every step of the TAQ cross-attention block runs in the library's
kernels. There is no CPU fallback: if the shared library is missing, loading
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtaq.so")

TAQ_OK = 0
TAQ_ERR_INVALID_ARG = -1
TAQ_ERR_UNSUPPORTED_BITS = -2
TAQ_ERR_BAD_SHAPE = -3
TAQ_ERR_MISALIGNED = -4
TAQ_ERR_HIP = -5
TAQ_ERR_SCRATCH_TOO_SMALL = -6
TAQ_STATIC_SCRATCH_BYTES = 16 << 20

TAQ_PROB_LINEAR = 0
TAQ_PROB_LOG2 = 1
TAQ_PROB_ROWMAX = 2

TAQ_STAGE_HIDDEN_QUANT = 1
TAQ_STAGE_TO_Q = 2
TAQ_STAGE_Q_QUANT = 4
TAQ_STAGE_ATTN_CORE = 8
TAQ_STAGE_O_QUANT = 16
TAQ_STAGE_TO_OUT = 32

EXPORTS = [
    "taq_kv_packed_bytes", "taq_kv_code_layout", "taq_workspace_bytes", "taq_quantize_weight", "taq_weight_bytes", "taq_pack_weight",
    "taq_quantize_kv",
    "taq_quantize_kv_w8",
    "taq_cross_attn", "taq_cross_attn_ex", "taq_cross_attn_static", "taq_cross_attn_batched", "taq_unpack_kv", "taq_mse_f16",
    "taq_status_string",
]


class TaqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {taq_status_string(status)} ({status})")


class taq_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("N", ctypes.c_int), ("C", ctypes.c_int), ("H", ctypes.c_int),
                ("T", ctypes.c_int), ("Cc", ctypes.c_int), ("bits_kv", ctypes.c_int),
                ("bits_prob", ctypes.c_int), ("bits_q", ctypes.c_int), ("bits_proj", ctypes.c_int),
                ("softmax_scale", ctypes.c_float), ("w_layout", ctypes.c_int), ("prob_grid", ctypes.c_int),
                ("tok_tile", ctypes.c_int)]


class taq_debug(ctypes.Structure):
    _fields_ = [("h_code", ctypes.c_void_p), ("s_h", ctypes.c_void_p), ("q_code", ctypes.c_void_p),
                ("s_Q", ctypes.c_void_p), ("O", ctypes.c_void_p), ("o_code", ctypes.c_void_p),
                ("s_o", ctypes.c_void_p), ("p_code", ctypes.c_void_p), ("stage_mask", ctypes.c_uint)]


class taq_request(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_void_p), ("qkv_packed", ctypes.c_void_p), ("Wq", ctypes.c_void_p),
                ("Wo", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("trigger_mask", ctypes.c_void_p),
                ("out", ctypes.c_void_p)]


_lib = None


def load() -> ctypes.CDLL:
    """Load libtaq.so (built by ``python -m paper_2603_22943_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_22943_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t), ctypes.c_int
    shp = ctypes.POINTER(taq_shape)
    lib.taq_status_string.restype = ctypes.c_char_p
    lib.taq_status_string.argtypes = [ci]
    lib.taq_kv_packed_bytes.argtypes = [shp, sz]
    lib.taq_workspace_bytes.argtypes = [shp, sz]
    lib.taq_kv_code_layout.argtypes = [shp, sz, sz, sz]
    lib.taq_quantize_weight.argtypes = [vp, ci, ci, vp, vp, vp]
    lib.taq_weight_bytes.argtypes = [shp, sz]
    lib.taq_pack_weight.argtypes = [vp, shp, vp, vp]
    lib.taq_quantize_kv.argtypes = [vp, vp, vp, vp, ci, shp, vp, vp, vp]
    lib.taq_quantize_kv_w8.argtypes = [vp, vp, vp, vp, ci, shp, vp, vp, vp]
    lib.taq_cross_attn.argtypes = [vp, vp, vp, vp, vp, vp, shp, vp, vp, vp]
    lib.taq_cross_attn_ex.argtypes = [vp, vp, vp, vp, vp, vp, shp, vp, vp, vp, ctypes.POINTER(taq_debug)]
    lib.taq_cross_attn_static.argtypes = [vp, vp, vp, vp, vp, vp, shp, vp, vp]
    lib.taq_cross_attn_batched.argtypes = [ci, ctypes.POINTER(taq_request), shp, vp, vp]
    lib.taq_unpack_kv.argtypes = [vp, shp, vp, vp, vp, vp, vp, vp, vp]
    lib.taq_mse_f16.argtypes = [vp, vp, ctypes.c_size_t, vp, vp]
    for name in EXPORTS:
        getattr(lib, name).restype = ctypes.c_char_p if name == "taq_status_string" else ci
    _lib = lib
    return lib


def make_shape(B: int, N: int, C: int, H: int, T: int, Cc: int, bits_kv: int = 8, bits_prob: int = 8,
               bits_q: int = 8, bits_proj: int = 8, softmax_scale: float = 0.0, w_layout: int = 0,
               prob_grid: int = 0, tok_tile: int = 0) -> taq_shape:
    return taq_shape(B, N, C, H, T, Cc, bits_kv, bits_prob, bits_q, bits_proj, softmax_scale, w_layout, prob_grid,
                     tok_tile)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(rc: int, where: str) -> None:
    if rc != TAQ_OK:
        raise TaqError(rc, where)


def taq_status_string(status: int) -> str:
    return load().taq_status_string(int(status)).decode()


def taq_kv_packed_bytes(shape: taq_shape) -> int:
    n = ctypes.c_size_t(0)
    _check(load().taq_kv_packed_bytes(ctypes.byref(shape), ctypes.byref(n)), "taq_kv_packed_bytes")
    return n.value


def taq_kv_code_layout(shape: taq_shape):
    """(byte offset of the K code section, of the V code section, bytes per (batch, token) row) inside qkv_packed."""
    k, v, rb = ctypes.c_size_t(0), ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load().taq_kv_code_layout(ctypes.byref(shape), ctypes.byref(k), ctypes.byref(v), ctypes.byref(rb)),
           "taq_kv_code_layout")
    return k.value, v.value, rb.value


def taq_workspace_bytes(shape: taq_shape) -> int:
    n = ctypes.c_size_t(0)
    _check(load().taq_workspace_bytes(ctypes.byref(shape), ctypes.byref(n)), "taq_workspace_bytes")
    return n.value


def taq_quantize_weight(W: torch.Tensor, codes: Optional[torch.Tensor] = None,
                        scales: Optional[torch.Tensor] = None, stream=None):
    """W f16 [rows, cols] on the GPU -> (int8 codes [rows, cols], f32 scales [rows])."""
    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous() and W.dim() == 2
    rows, cols = W.shape
    if codes is None:
        codes = torch.empty((rows, cols), dtype=torch.int8, device=W.device)
    if scales is None:
        scales = torch.empty((rows,), dtype=torch.float32, device=W.device)
    _check(load().taq_quantize_weight(_ptr(W), rows, cols, _ptr(codes), _ptr(scales), _stream(stream)),
           "taq_quantize_weight")
    return codes, scales


def taq_weight_bytes(shape: taq_shape) -> int:
    n = ctypes.c_size_t(0)
    _check(load().taq_weight_bytes(ctypes.byref(shape), ctypes.byref(n)), "taq_weight_bytes")
    return n.value


def taq_pack_weight(codes: torch.Tensor, shape: taq_shape, out: Optional[torch.Tensor] = None, stream=None):
    """int8 [C, C] row-major codes -> buffer for taq_cross_attn with shape.w_layout = 1."""
    if out is None:
        out = torch.empty(taq_weight_bytes(shape), dtype=torch.int8, device=codes.device)
    _check(load().taq_pack_weight(_ptr(codes), ctypes.byref(shape), _ptr(out), _stream(stream)), "taq_pack_weight")
    return out


def taq_quantize_kv(context: torch.Tensor, trigger_mask: torch.Tensor, Wk: torch.Tensor, Wv: torch.Tensor,
                    bits: int, shape: taq_shape, qkv_packed: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Eq. (2), K and V lines. Returns the opaque qkv_packed byte tensor."""
    dev = context.device
    if qkv_packed is None:
        qkv_packed = torch.empty(taq_kv_packed_bytes(shape), dtype=torch.uint8, device=dev)
    if workspace is None:
        workspace = torch.empty(taq_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    _check(load().taq_quantize_kv(_ptr(context), _ptr(trigger_mask), _ptr(Wk), _ptr(Wv), int(bits),
                                  ctypes.byref(shape), _ptr(qkv_packed), _ptr(workspace), _stream(stream)),
           "taq_quantize_kv")
    return qkv_packed


def taq_quantize_kv_w8(context: torch.Tensor, trigger_mask: torch.Tensor, Wkv_code: torch.Tensor, s_wkv: torch.Tensor,
                       bits: int, shape: taq_shape, qkv_packed: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """taq_quantize_kv with the weight codes of to_k / to_v (int8 [2C, Cc], f32 [2C]) formed beforehand."""
    dev = context.device
    if qkv_packed is None:
        qkv_packed = torch.empty(taq_kv_packed_bytes(shape), dtype=torch.uint8, device=dev)
    if workspace is None:
        workspace = torch.empty(taq_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    _check(load().taq_quantize_kv_w8(_ptr(context), _ptr(trigger_mask), _ptr(Wkv_code), _ptr(s_wkv), int(bits),
                                     ctypes.byref(shape), _ptr(qkv_packed), _ptr(workspace), _stream(stream)),
           "taq_quantize_kv_w8")
    return qkv_packed


def taq_cross_attn(hidden: torch.Tensor, qkv_packed: torch.Tensor, Wq: torch.Tensor, Wo: torch.Tensor,
                   scales: torch.Tensor, trigger_mask: Optional[torch.Tensor], shape: taq_shape,
                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                   stream=None, debug: Optional[taq_debug] = None) -> torch.Tensor:
    """The TAQ block for image tokens; returns out f16 [B, N, C]."""
    dev = hidden.device
    if out is None:
        out = torch.empty((shape.B, shape.N, shape.C), dtype=torch.float16, device=dev)
    if workspace is None:
        workspace = torch.empty(taq_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    lib = load()
    if debug is None:
        rc = lib.taq_cross_attn(_ptr(hidden), _ptr(qkv_packed), _ptr(Wq), _ptr(Wo), _ptr(scales),
                                _ptr(trigger_mask), ctypes.byref(shape), _ptr(out), _ptr(workspace),
                                _stream(stream))
    else:
        rc = lib.taq_cross_attn_ex(_ptr(hidden), _ptr(qkv_packed), _ptr(Wq), _ptr(Wo), _ptr(scales),
                                   _ptr(trigger_mask), ctypes.byref(shape), _ptr(out), _ptr(workspace),
                                   _stream(stream), ctypes.byref(debug))
    _check(rc, "taq_cross_attn")
    return out


def taq_cross_attn_static(hidden: torch.Tensor, qkv_packed: torch.Tensor, Wq: torch.Tensor, Wo: torch.Tensor,
                          scales: torch.Tensor, trigger_mask: Optional[torch.Tensor], shape: taq_shape,
                          out: torch.Tensor, stream=None) -> torch.Tensor:
    """taq_cross_attn on the library's static scratch array: no workspace argument, nothing allocated (the
    caller passes `out`)."""
    _check(load().taq_cross_attn_static(_ptr(hidden), _ptr(qkv_packed), _ptr(Wq), _ptr(Wo), _ptr(scales),
                                        _ptr(trigger_mask), ctypes.byref(shape), _ptr(out), _stream(stream)),
           "taq_cross_attn_static")
    return out


def taq_cross_attn_batched(requests: Sequence[dict], shape: taq_shape, workspace: Optional[torch.Tensor] = None,
                           stream=None) -> None:
    """requests: dicts with tensors hidden, qkv_packed, Wq, Wo, scales, trigger_mask (or None), out."""
    R = len(requests)
    table = (taq_request * max(R, 1))()
    for r, q in enumerate(requests):
        table[r] = taq_request(_ptr(q["hidden"]), _ptr(q["qkv_packed"]), _ptr(q["Wq"]), _ptr(q["Wo"]),
                               _ptr(q["scales"]), _ptr(q.get("trigger_mask")), _ptr(q["out"]))
    if workspace is None:
        workspace = torch.empty(max(R, 1) * taq_workspace_bytes(shape), dtype=torch.uint8,
                                device=requests[0]["hidden"].device if R else "cuda")
    _check(load().taq_cross_attn_batched(R, table, ctypes.byref(shape), _ptr(workspace), _stream(stream)),
           "taq_cross_attn_batched")


def taq_mse_f16(x: torch.Tensor, y: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Mean squared difference of two fp16 tensors of equal size -> float64 tensor of one element on the device."""
    assert x.dtype == torch.float16 and y.dtype == torch.float16 and x.numel() == y.numel()
    assert x.is_contiguous() and y.is_contiguous()
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=x.device)
    _check(load().taq_mse_f16(_ptr(x), _ptr(y), x.numel(), _ptr(out), _stream(stream)), "taq_mse_f16")
    return out


def taq_unpack_kv(qkv_packed: torch.Tensor, shape: taq_shape, stream=None) -> dict:
    """Expand qkv_packed into plain tensors (tests)."""
    dev = qkv_packed.device
    B, T, C, H = shape.B, shape.T, shape.C, shape.H
    out = dict(
        k_code=torch.empty((B, T, C), dtype=torch.int8, device=dev),
        v_code=torch.empty((B, T, C), dtype=torch.int8, device=dev),
        s_K=torch.empty((B, H, T), dtype=torch.float32, device=dev),
        s_V=torch.empty((B, H, T), dtype=torch.float32, device=dev),
        K16=torch.empty((B, T, C), dtype=torch.float16, device=dev),
        V16=torch.empty((B, T, C), dtype=torch.float16, device=dev),
    )
    _check(load().taq_unpack_kv(_ptr(qkv_packed), ctypes.byref(shape), _ptr(out["k_code"]), _ptr(out["v_code"]),
                                _ptr(out["s_K"]), _ptr(out["s_V"]), _ptr(out["K16"]), _ptr(out["V16"]),
                                _stream(stream)), "taq_unpack_kv")
    return out


def make_debug(shape: taq_shape, device, stage_mask: int = 0, taps: bool = True):
    """Allocate tap tensors for taq_cross_attn(debug=...). Returns (taq_debug, dict of tensors)."""
    M = shape.B * shape.N
    t = {}
    if taps:
        t = dict(
            h_code=torch.empty((shape.B, shape.N, shape.C), dtype=torch.int8, device=device),
            s_h=torch.empty((shape.B, shape.N), dtype=torch.float32, device=device),
            q_code=torch.empty((shape.B, shape.N, shape.C), dtype=torch.int8, device=device),
            s_Q=torch.empty((shape.B, shape.N, shape.H), dtype=torch.float32, device=device),
            O=torch.empty((shape.B, shape.N, shape.C), dtype=torch.float32, device=device),
            o_code=torch.empty((shape.B, shape.N, shape.C), dtype=torch.int8, device=device),
            s_o=torch.empty((shape.B, shape.N), dtype=torch.float32, device=device),
            p_code=torch.zeros((shape.B, shape.N, shape.H, shape.T), dtype=torch.uint8, device=device),
        )
    dbg = taq_debug(_ptr(t.get("h_code")), _ptr(t.get("s_h")), _ptr(t.get("q_code")), _ptr(t.get("s_Q")),
                    _ptr(t.get("O")), _ptr(t.get("o_code")), _ptr(t.get("s_o")), _ptr(t.get("p_code")), stage_mask)
    return dbg, t
