"""ctypes binding of libqail.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/qail.h) and
takes torch tensors that already live on the GPU; torch is used for device
memory and for the current stream, nothing else.  There is no fallback: if the
library has not been built, or a call returns an error status, an exception is
raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqail.so")

QAIL_W4_ASYM_GROUP = 0
QAIL_W4_SYM_CHANNEL = 1

QAIL_OK = 0
QAIL_ERR_NULL = -1
QAIL_ERR_SHAPE = -2
QAIL_ERR_ALIGN = -3
QAIL_ERR_WORKSPACE = -4
QAIL_ERR_UNSUPPORTED = -5
QAIL_ERR_HIP = -6

EXPORTS = (
    "qail_version", "qail_status_string", "qail_packed_sizes", "qail_quantize_weights",
    "qail_unpack_weights", "qail_act_scale_u4", "qail_quantize_act_u4", "qail_w4a16_workspace",
    "qail_w4a16_linear", "qail_w4a16_linear_batch", "qail_w4a16_batch_workspace",
    "qail_w4a4_workspace", "qail_w4a4_gemm", "qail_w4a4_conv_u4", "qail_w4a4_conv_batch",
    "qail_w4a16_lora_workspace", "qail_w4a16_linear_lora_batch",
    "qail_static_scratch_bytes", "qail_w4a16_linear_lora_batch_static",
    "qail_w4a16_chain_workspace", "qail_w4a16_linear_chain",
    "qail_act_scale_s8", "qail_quantize_act_s8", "qail_w8a8_gemm", "qail_w8a16_linear",
    "qail_w8a16_linear_batch", "qail_w8a16_workspace", "qail_w8a16_batch_workspace",
    "qail_fake_quant_w4", "qail_lsq_forward", "qail_lsq_backward_workspace", "qail_lsq_backward", "qail_qbc_loss",
)


class QailError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class qail_lora(ctypes.Structure):
    _fields_ = [("A", ctypes.c_void_p), ("B", ctypes.c_void_p), ("r", ctypes.c_int32), ("scaling", ctypes.c_float)]


class qail_wdesc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("K", ctypes.c_int32), ("group_size", ctypes.c_int32),
                ("scheme", ctypes.c_int32)]


class qail_conv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "H", "W", "Cin", "Cout", "KH", "KW", "stride", "pad")]


class qail_conv_item(ctypes.Structure):
    _fields_ = [("d", qail_conv_desc), ("a_u4", ctypes.c_void_p), ("w_s4", ctypes.c_void_p),
                ("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("acc_out", ctypes.c_void_p),
                ("y_out", ctypes.c_void_p), ("out_u4", ctypes.c_void_p), ("s_out", ctypes.c_float),
                ("res_scale", ctypes.c_float), ("res_u4", ctypes.c_void_p), ("res_f32", ctypes.c_void_p)]


class qail_w4a16_item(ctypes.Structure):
    _fields_ = [("d", qail_wdesc), ("qweight", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("zeros", ctypes.c_void_p), ("x", ctypes.c_void_p), ("y", ctypes.c_void_p)]


class qail_w8a16_item(ctypes.Structure):
    _fields_ = [("d", qail_wdesc), ("qweight", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("x", ctypes.c_void_p), ("y", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2412_01034_amd.build)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
        psz = ctypes.POINTER(ctypes.c_size_t)
        L.qail_version.restype = ctypes.c_int
        L.qail_version.argtypes = []
        L.qail_status_string.restype = ctypes.c_char_p
        L.qail_status_string.argtypes = [ctypes.c_int]
        L.qail_packed_sizes.argtypes = [ctypes.POINTER(qail_wdesc), psz, psz, psz]
        L.qail_quantize_weights.argtypes = [ctypes.POINTER(qail_wdesc), vp, vp, vp, vp, vp, vp]
        L.qail_unpack_weights.argtypes = [ctypes.POINTER(qail_wdesc), vp, vp, vp]
        L.qail_act_scale_u4.argtypes = [vp, sz, vp, vp]
        L.qail_quantize_act_u4.argtypes = [vp, sz, vp, vp, vp]
        L.qail_w4a16_workspace.argtypes = [ctypes.POINTER(qail_wdesc), i32, psz]
        L.qail_w4a16_linear.argtypes = [ctypes.POINTER(qail_wdesc), vp, vp, vp, vp, vp, i32, vp, sz, vp]
        L.qail_w4a16_linear_batch.argtypes = [ctypes.POINTER(qail_w4a16_item), i32, i32, vp, sz, vp]
        L.qail_w4a16_batch_workspace.argtypes = [ctypes.POINTER(qail_w4a16_item), i32, i32, psz]
        L.qail_w4a16_lora_workspace.argtypes = [ctypes.POINTER(qail_w4a16_item), ctypes.POINTER(qail_lora), i32, i32, psz]
        L.qail_w4a16_linear_lora_batch.argtypes = [ctypes.POINTER(qail_w4a16_item), ctypes.POINTER(qail_lora), i32,
                                                   i32, vp, sz, vp]
        L.qail_static_scratch_bytes.argtypes = [psz]
        L.qail_w4a16_chain_workspace.argtypes = [ctypes.POINTER(qail_w4a16_item), i32, psz]
        L.qail_w4a16_linear_chain.argtypes = [ctypes.POINTER(qail_w4a16_item), i32, vp, sz, vp]
        L.qail_w4a16_linear_lora_batch_static.argtypes = [ctypes.POINTER(qail_w4a16_item), ctypes.POINTER(qail_lora),
                                                          i32, i32, vp]
        L.qail_fake_quant_w4.argtypes = [ctypes.POINTER(qail_wdesc), vp, vp, vp]
        L.qail_lsq_forward.argtypes = [vp, sz, vp, i32, i32, vp, vp]
        L.qail_lsq_backward_workspace.argtypes = [psz]
        L.qail_lsq_backward.argtypes = [vp, vp, sz, vp, i32, i32, ctypes.c_float, vp, vp, vp, sz, vp]
        L.qail_qbc_loss.argtypes = [vp, vp, i32, i32, vp, vp, vp, sz, vp]
        L.qail_act_scale_s8.argtypes = [vp, sz, vp, vp]
        L.qail_quantize_act_s8.argtypes = [vp, sz, vp, vp, vp]
        L.qail_w8a8_gemm.argtypes = [ctypes.POINTER(qail_conv_desc), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.qail_w8a16_linear.argtypes = [ctypes.POINTER(qail_wdesc), vp, vp, vp, vp, i32, vp, sz, vp]
        L.qail_w8a16_workspace.argtypes = [ctypes.POINTER(qail_wdesc), i32, psz]
        L.qail_w8a16_batch_workspace.argtypes = [ctypes.POINTER(qail_w8a16_item), i32, i32, psz]
        L.qail_w8a16_linear_batch.argtypes = [ctypes.POINTER(qail_w8a16_item), i32, i32, vp, sz, vp]
        L.qail_w4a4_workspace.argtypes = [ctypes.POINTER(qail_conv_desc), psz]
        L.qail_w4a4_gemm.argtypes = [ctypes.POINTER(qail_conv_desc), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.qail_w4a4_conv_batch.argtypes = [ctypes.POINTER(qail_conv_item), i32, vp]
        L.qail_w4a4_conv_u4.argtypes = [ctypes.POINTER(qail_conv_desc), vp, vp, vp, vp, ctypes.c_float, vp,
                                        ctypes.c_float, vp, vp, vp, sz, vp]
        for name in EXPORTS:
            if name not in ("qail_status_string",):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().qail_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != QAIL_OK:
        raise QailError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _need(t: torch.Tensor, nbytes: int, what: str) -> None:
    if t.numel() * t.element_size() < nbytes:
        raise ValueError(f"{what}: {t.numel() * t.element_size()} bytes given, {nbytes} needed")


def qail_version() -> int:
    return int(lib().qail_version())


def qail_packed_sizes(N: int, K: int, group_size: int, scheme: int) -> Tuple[int, int, int]:
    d = qail_wdesc(N, K, group_size, scheme)
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().qail_packed_sizes(ctypes.byref(d), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)),
           "qail_packed_sizes")
    return a.value, b.value, c.value


def qail_quantize_weights(w: torch.Tensor, group_size: int, scheme: int, qweight: torch.Tensor,
                          scales: torch.Tensor, zeros: Optional[torch.Tensor],
                          range_errors: Optional[torch.Tensor] = None) -> None:
    """w: fp32 [N, K] (any leading shape whose product is N for SYM_CHANNEL's
    [Cout, KH, KW, Cin]); outputs are preallocated device tensors."""
    N = w.shape[0]
    K = w.numel() // N
    if w.dtype != torch.float32:
        raise ValueError("fp32 weights expected")
    qb, sb, zb = qail_packed_sizes(N, K, group_size, scheme)
    _need(qweight, qb, "qweight")
    _need(scales, sb, "scales")
    if zb:
        if zeros is None:
            raise ValueError("zeros required")
        _need(zeros, zb, "zeros")
    d = qail_wdesc(N, K, group_size, scheme)
    _check(lib().qail_quantize_weights(ctypes.byref(d), _ptr(w), _ptr(qweight), _ptr(scales), _ptr(zeros),
                                       _ptr(range_errors), _stream()), "qail_quantize_weights")


def qail_unpack_weights(N: int, K: int, group_size: int, scheme: int, qweight: torch.Tensor,
                        codes: torch.Tensor) -> None:
    _need(qweight, N * K // 2, "qweight")
    _need(codes, N * K, "codes")
    d = qail_wdesc(N, K, group_size, scheme)
    _check(lib().qail_unpack_weights(ctypes.byref(d), _ptr(qweight), _ptr(codes), _stream()),
           "qail_unpack_weights")


def qail_act_scale_u4(a: torch.Tensor, s_a: torch.Tensor) -> None:
    if a.dtype != torch.float32 or s_a.dtype != torch.float32:
        raise ValueError("fp32 expected")
    _check(lib().qail_act_scale_u4(_ptr(a) if a.numel() else None, a.numel(), _ptr(s_a), _stream()),
           "qail_act_scale_u4")


def qail_quantize_act_u4(a: torch.Tensor, s_a: torch.Tensor, a_u4: torch.Tensor) -> None:
    if a.dtype != torch.float32 or s_a.dtype != torch.float32:
        raise ValueError("fp32 expected")
    _need(a_u4, a.numel() // 2, "a_u4")
    _check(lib().qail_quantize_act_u4(_ptr(a) if a.numel() else None, a.numel(), _ptr(s_a),
                                      _ptr(a_u4) if a.numel() else None, _stream()), "qail_quantize_act_u4")


def qail_w4a16_workspace(N: int, K: int, group_size: int, M: int) -> int:
    d = qail_wdesc(N, K, group_size, QAIL_W4_ASYM_GROUP)
    b = ctypes.c_size_t()
    _check(lib().qail_w4a16_workspace(ctypes.byref(d), M, ctypes.byref(b)), "qail_w4a16_workspace")
    return b.value


def qail_w4a16_linear(N: int, K: int, group_size: int, qweight: torch.Tensor, scales: torch.Tensor,
                      zeros: torch.Tensor, x: torch.Tensor, y: torch.Tensor, M: int,
                      workspace: Optional[torch.Tensor] = None) -> None:
    """x: bf16 [M, K]; y: bf16 [M, N]; both device tensors (torch.bfloat16 or a
    16-bit integer view of the same bits)."""
    G = K // group_size
    _need(qweight, N * K // 2, "qweight")
    _need(scales, N * G * 2, "scales")
    _need(zeros, N * ((G + 7) // 8) * 4, "zeros")
    _need(x, M * K * 2, "x")
    _need(y, M * N * 2, "y")
    d = qail_wdesc(N, K, group_size, QAIL_W4_ASYM_GROUP)
    wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().qail_w4a16_linear(ctypes.byref(d), _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(x),
                                   _ptr(y), M, _ptr(workspace), wsb, _stream()), "qail_w4a16_linear")


def make_w4a16_items(entries: Sequence[dict], M: int):
    """entries: dicts with N, K, group_size, qweight, scales, zeros, x, y (device
    tensors).  Returns a ctypes array that can be passed to qail_w4a16_linear_batch
    any number of times (the tensors must be kept alive by the caller)."""
    arr = (qail_w4a16_item * max(1, len(entries)))()
    for i, e in enumerate(entries):
        N, K, g = e["N"], e["K"], e["group_size"]
        G = K // g
        _need(e["qweight"], N * K // 2, "qweight")
        _need(e["scales"], N * G * 2, "scales")
        _need(e["zeros"], N * ((G + 7) // 8) * 4, "zeros")
        _need(e["x"], M * K * 2, "x")
        _need(e["y"], M * N * 2, "y")
        arr[i].d = qail_wdesc(N, K, g, QAIL_W4_ASYM_GROUP)
        arr[i].qweight = _ptr(e["qweight"])
        arr[i].scales = _ptr(e["scales"])
        arr[i].zeros = _ptr(e["zeros"])
        arr[i].x = _ptr(e["x"])
        arr[i].y = _ptr(e["y"])
    return arr


def qail_w4a16_batch_workspace(items, count: int, M: int) -> int:
    b = ctypes.c_size_t()
    _check(lib().qail_w4a16_batch_workspace(items, count, M, ctypes.byref(b)), "qail_w4a16_batch_workspace")
    return b.value


def qail_w4a16_linear_batch(items, count: int, M: int, workspace: Optional[torch.Tensor] = None,
                            stream: Optional[int] = None) -> None:
    wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().qail_w4a16_linear_batch(items, count, M, _ptr(workspace), wsb,
                                         _stream() if stream is None else stream), "qail_w4a16_linear_batch")


def qail_w4a4_workspace(B, H, W, Cin, Cout, KH, KW, stride, pad) -> int:
    d = qail_conv_desc(B, H, W, Cin, Cout, KH, KW, stride, pad)
    b = ctypes.c_size_t()
    _check(lib().qail_w4a4_workspace(ctypes.byref(d), ctypes.byref(b)), "qail_w4a4_workspace")
    return b.value


def qail_w4a4_gemm(B, H, W, Cin, Cout, KH, KW, stride, pad, a_u4: torch.Tensor, w_s4: torch.Tensor,
                   acc_out: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None,
                   bias: Optional[torch.Tensor] = None, y_out: Optional[torch.Tensor] = None,
                   workspace: Optional[torch.Tensor] = None, stream: Optional[int] = None) -> None:
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    M = B * OH * OW
    _need(a_u4, B * H * W * Cin // 2, "a_u4")
    _need(w_s4, Cout * KH * KW * Cin // 2, "w_s4")
    if acc_out is not None:
        _need(acc_out, M * Cout * 4, "acc_out")
    if y_out is not None:
        _need(y_out, M * Cout * 4, "y_out")
    for t, nm in ((scale, "scale"), (bias, "bias")):
        if t is not None:
            _need(t, Cout * 4, nm)
    d = qail_conv_desc(B, H, W, Cin, Cout, KH, KW, stride, pad)
    wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().qail_w4a4_gemm(ctypes.byref(d), _ptr(a_u4), _ptr(w_s4), _ptr(acc_out), _ptr(scale),
                                _ptr(bias), _ptr(y_out), _ptr(workspace), wsb,
                                _stream() if stream is None else stream), "qail_w4a4_gemm")


def qail_w4a4_conv_u4(B, H, W, Cin, Cout, KH, KW, stride, pad, a_u4: torch.Tensor, w_s4: torch.Tensor,
                      scale: torch.Tensor, bias: torch.Tensor, s_out: float, out_u4: torch.Tensor,
                      res_u4: Optional[torch.Tensor] = None, res_scale: float = 0.0,
                      res_f32: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                      stream: Optional[int] = None) -> None:
    """Convolution with the fused 4-bit output epilogue; out_u4: [M, Cout/8] packed words."""
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    M = B * OH * OW
    _need(a_u4, B * H * W * Cin // 2, "a_u4")
    _need(w_s4, Cout * KH * KW * Cin // 2, "w_s4")
    _need(scale, Cout * 4, "scale")
    _need(bias, Cout * 4, "bias")
    _need(out_u4, M * Cout // 2, "out_u4")
    if res_u4 is not None:
        _need(res_u4, M * Cout // 2, "res_u4")
    if res_f32 is not None:
        _need(res_f32, M * Cout * 4, "res_f32")
    d = qail_conv_desc(B, H, W, Cin, Cout, KH, KW, stride, pad)
    wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().qail_w4a4_conv_u4(ctypes.byref(d), _ptr(a_u4), _ptr(w_s4), _ptr(scale), _ptr(bias),
                                   float(s_out), _ptr(res_u4), float(res_scale), _ptr(res_f32), _ptr(out_u4),
                                   _ptr(workspace), wsb, _stream() if stream is None else stream),
           "qail_w4a4_conv_u4")


def make_conv_items(entries: Sequence[dict]):
    """entries: dicts with the conv fields B, H, W, Cin, Cout, KH, KW, stride, pad, the device tensors a_u4,
    w_s4 and, as the item needs them, scale, bias, acc_out, y_out, out_u4, res_u4, res_f32, and the host
    values s_out, res_scale.  The tensors must be kept alive by the caller."""
    arr = (qail_conv_item * max(1, len(entries)))()
    for i, e in enumerate(entries):
        B, H, W, Cin, Cout, KH, KW, stride, pad = (int(e[k]) for k in ("B", "H", "W", "Cin", "Cout", "KH", "KW", "stride", "pad"))
        M = B * ((H + 2 * pad - KH) // stride + 1) * ((W + 2 * pad - KW) // stride + 1)
        _need(e["a_u4"], B * H * W * Cin // 2, "a_u4")
        _need(e["w_s4"], Cout * KH * KW * Cin // 2, "w_s4")
        for name, nbytes in (("scale", Cout * 4), ("bias", Cout * 4), ("acc_out", M * Cout * 4), ("y_out", M * Cout * 4),
                             ("out_u4", M * Cout // 2), ("res_u4", M * Cout // 2), ("res_f32", M * Cout * 4)):
            if e.get(name) is not None:
                _need(e[name], nbytes, name)
        arr[i] = qail_conv_item(qail_conv_desc(B, H, W, Cin, Cout, KH, KW, stride, pad), _ptr(e["a_u4"]), _ptr(e["w_s4"]),
                                _ptr(e.get("scale")), _ptr(e.get("bias")), _ptr(e.get("acc_out")), _ptr(e.get("y_out")),
                                _ptr(e.get("out_u4")), float(e.get("s_out", 0.0)), float(e.get("res_scale", 0.0)),
                                _ptr(e.get("res_u4")), _ptr(e.get("res_f32")))
    return arr


def qail_w4a4_conv_batch(items, count: int, stream: Optional[int] = None) -> None:
    _check(lib().qail_w4a4_conv_batch(items, count, _stream() if stream is None else stream), "qail_w4a4_conv_batch")


def make_loras(entries: Sequence[dict]):
    """entries: dicts with A (bf16 [r, K]), B (bf16 [N, r]) device tensors, r, scaling, and the
    linear's N and K for the size check.  The tensors must be kept alive by the caller."""
    arr = (qail_lora * max(1, len(entries)))()
    for i, e in enumerate(entries):
        _need(e["A"], e["r"] * e["K"] * 2, "A")
        _need(e["B"], e["N"] * e["r"] * 2, "B")
        arr[i] = qail_lora(_ptr(e["A"]), _ptr(e["B"]), int(e["r"]), float(e["scaling"]))
    return arr


def qail_w4a16_lora_workspace(items, loras, count: int, M: int) -> int:
    b = ctypes.c_size_t()
    _check(lib().qail_w4a16_lora_workspace(items, loras, count, M, ctypes.byref(b)), "qail_w4a16_lora_workspace")
    return b.value


def qail_w4a16_linear_lora_batch(items, loras, count: int, M: int, workspace: torch.Tensor,
                                 stream: Optional[int] = None) -> None:
    wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().qail_w4a16_linear_lora_batch(items, loras, count, M, _ptr(workspace), wsb,
                                              _stream() if stream is None else stream),
           "qail_w4a16_linear_lora_batch")


def qail_w4a16_chain_workspace(items, count: int) -> int:
    b = ctypes.c_size_t()
    _check(lib().qail_w4a16_chain_workspace(items, count, ctypes.byref(b)), "qail_w4a16_chain_workspace")
    return b.value


def qail_w4a16_linear_chain(items, count: int, workspace: torch.Tensor, stream: Optional[int] = None) -> None:
    wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().qail_w4a16_linear_chain(items, count, _ptr(workspace), wsb, _stream() if stream is None else stream),
           "qail_w4a16_linear_chain")


def qail_static_scratch_bytes() -> int:
    b = ctypes.c_size_t()
    _check(lib().qail_static_scratch_bytes(ctypes.byref(b)), "qail_static_scratch_bytes")
    return b.value


def qail_w4a16_linear_lora_batch_static(items, loras, count: int, M: int, stream: Optional[int] = None) -> None:
    _check(lib().qail_w4a16_linear_lora_batch_static(items, loras, count, M, _stream() if stream is None else stream),
           "qail_w4a16_linear_lora_batch_static")


QAIL_W8_SYM_CHANNEL = 2
QAIL_W8_SYM_GROUP = 3


def qail_act_scale_s8(a: torch.Tensor, s_a: torch.Tensor) -> None:
    _need(a, a.numel() * 4, "a")
    _check(lib().qail_act_scale_s8(_ptr(a), a.numel(), _ptr(s_a), _stream()), "qail_act_scale_s8")


def qail_quantize_act_s8(a: torch.Tensor, s_a: torch.Tensor, a_s8: torch.Tensor) -> None:
    _need(a_s8, a.numel(), "a_s8")
    _check(lib().qail_quantize_act_s8(_ptr(a), a.numel(), _ptr(s_a), _ptr(a_s8), _stream()), "qail_quantize_act_s8")


def qail_w8a8_gemm(B, H, W, Cin, Cout, KH, KW, stride, pad, a_s8: torch.Tensor, w_s8: torch.Tensor,
                   acc_out: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None,
                   bias: Optional[torch.Tensor] = None, y_out: Optional[torch.Tensor] = None,
                   stream: Optional[int] = None) -> None:
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    M = B * OH * OW
    _need(a_s8, B * H * W * Cin, "a_s8")
    _need(w_s8, Cout * KH * KW * Cin, "w_s8")
    for t, nm in ((acc_out, "acc_out"), (y_out, "y_out")):
        if t is not None:
            _need(t, M * Cout * 4, nm)
    d = qail_conv_desc(B, H, W, Cin, Cout, KH, KW, stride, pad)
    _check(lib().qail_w8a8_gemm(ctypes.byref(d), _ptr(a_s8), _ptr(w_s8), _ptr(acc_out), _ptr(scale), _ptr(bias),
                                _ptr(y_out), None, 0, _stream() if stream is None else stream), "qail_w8a8_gemm")


def qail_w8a16_workspace(N: int, K: int, group_size: int, M: int) -> int:
    d = qail_wdesc(N, K, group_size, QAIL_W8_SYM_GROUP)
    b = ctypes.c_size_t()
    _check(lib().qail_w8a16_workspace(ctypes.byref(d), M, ctypes.byref(b)), "qail_w8a16_workspace")
    return b.value


def qail_w8a16_linear(N: int, K: int, group_size: int, qweight: torch.Tensor, scales: torch.Tensor,
                      x: torch.Tensor, y: torch.Tensor, M: int, workspace: Optional[torch.Tensor] = None,
                      stream: Optional[int] = None) -> None:
    _need(qweight, N * K, "qweight")
    _need(scales, N * (K // group_size) * 2, "scales")
    _need(x, M * K * 2, "x")
    _need(y, M * N * 2, "y")
    d = qail_wdesc(N, K, group_size, QAIL_W8_SYM_GROUP)
    wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().qail_w8a16_linear(ctypes.byref(d), _ptr(qweight), _ptr(scales), _ptr(x), _ptr(y), M,
                                   _ptr(workspace), wsb, _stream() if stream is None else stream), "qail_w8a16_linear")


def make_w8a16_items(entries: Sequence[dict], M: int):
    """entries: dicts with N, K, group_size, qweight, scales, x, y (device tensors).  Returns a ctypes
    array for qail_w8a16_linear_batch (the tensors must be kept alive by the caller)."""
    arr = (qail_w8a16_item * max(1, len(entries)))()
    for i, e in enumerate(entries):
        N, K, g = e["N"], e["K"], e["group_size"]
        _need(e["qweight"], N * K, "qweight")
        _need(e["scales"], N * (K // g) * 2, "scales")
        _need(e["x"], M * K * 2, "x")
        _need(e["y"], M * N * 2, "y")
        arr[i].d = qail_wdesc(N, K, g, QAIL_W8_SYM_GROUP)
        arr[i].qweight = _ptr(e["qweight"])
        arr[i].scales = _ptr(e["scales"])
        arr[i].x = _ptr(e["x"])
        arr[i].y = _ptr(e["y"])
    return arr


def qail_w8a16_batch_workspace(items, count: int, M: int) -> int:
    b = ctypes.c_size_t()
    _check(lib().qail_w8a16_batch_workspace(items, count, M, ctypes.byref(b)), "qail_w8a16_batch_workspace")
    return b.value


def qail_w8a16_linear_batch(items, count: int, M: int, workspace: Optional[torch.Tensor] = None,
                            stream: Optional[int] = None) -> None:
    wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().qail_w8a16_linear_batch(items, count, M, _ptr(workspace), wsb,
                                         _stream() if stream is None else stream), "qail_w8a16_linear_batch")


def qail_fake_quant_w4(w: torch.Tensor, group_size: int, w_hat: torch.Tensor) -> None:
    N = w.shape[0]
    K = w.numel() // N
    _need(w_hat, N * K * 4, "w_hat")
    d = qail_wdesc(N, K, group_size, QAIL_W4_ASYM_GROUP)
    _check(lib().qail_fake_quant_w4(ctypes.byref(d), _ptr(w), _ptr(w_hat), _stream()), "qail_fake_quant_w4")


def qail_lsq_forward(v: torch.Tensor, s: torch.Tensor, qn: int, qp: int, v_hat: torch.Tensor) -> None:
    _need(v_hat, v.numel() * 4, "v_hat")
    _check(lib().qail_lsq_forward(_ptr(v), v.numel(), _ptr(s), qn, qp, _ptr(v_hat), _stream()), "qail_lsq_forward")


def qail_lsq_backward(v: torch.Tensor, dout: torch.Tensor, s: torch.Tensor, qn: int, qp: int, grad_scale: float,
                      dv: torch.Tensor, ds: torch.Tensor, workspace: torch.Tensor) -> None:
    _need(dout, v.numel() * 4, "dout")
    _need(dv, v.numel() * 4, "dv")
    _check(lib().qail_lsq_backward(_ptr(v), _ptr(dout), v.numel(), _ptr(s), qn, qp, float(grad_scale), _ptr(dv),
                                   _ptr(ds), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "qail_lsq_backward")


def qail_lsq_backward_workspace() -> int:
    b = ctypes.c_size_t()
    _check(lib().qail_lsq_backward_workspace(ctypes.byref(b)), "qail_lsq_backward_workspace")
    return b.value


def qail_qbc_loss(logits_q: torch.Tensor, logits_fp: torch.Tensor, loss: torch.Tensor,
                  grad_q: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    Bn, D = logits_q.shape
    _need(logits_fp, Bn * D * 4, "logits_fp")
    if grad_q is not None:
        _need(grad_q, Bn * D * 4, "grad_q")
    _check(lib().qail_qbc_loss(_ptr(logits_q), _ptr(logits_fp), Bn, D, _ptr(loss), _ptr(grad_q), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream()), "qail_qbc_loss")
