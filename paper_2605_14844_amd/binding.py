"""ctypes binding of libxfp.so with the same entry-point names as include/xfp.h.

Argument marshalling only: tensors are passed as raw device pointers and the
current torch stream as a hipStream_t.  Every computation runs in the HIP
kernels behind the C ABI.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

XFP_MODE_V2, XFP_MODE_V2A = 0, 1
XFP_F16, XFP_F32, XFP_BF16 = 0, 1, 2
XFP_X_BF16 = 0x100
XFP_CHECK_GROUP_ID, XFP_CHECK_ROW_PTR, XFP_CHECK_COL_RANGE, XFP_CHECK_COL_ORDER, XFP_CHECK_EXPERT_ID = 1, 2, 3, 4, 5

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libxfp.so")
_lib = None


class XfpError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"xfp status {status}: {text}")
        self.status = status


class xfp_weights(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32), ("mode", ctypes.c_uint32), ("bits", ctypes.c_uint32),
        ("group", ctypes.c_uint32), ("N", ctypes.c_uint32), ("K", ctypes.c_uint32),
        ("L", ctypes.c_uint32), ("E", ctypes.c_uint32), ("flags", ctypes.c_uint32),
        ("reserved", ctypes.c_uint32),
        ("indices", ctypes.c_void_p), ("codebooks", ctypes.c_void_p), ("group_ids", ctypes.c_void_p),
        ("out_row_ptr", ctypes.c_void_p), ("out_col", ctypes.c_void_p), ("out_val", ctypes.c_void_p),
        ("group_scale", ctypes.c_void_p), ("group_mid", ctypes.c_void_p),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libxfp.so; build it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("XFP_LIBRARY", _LIB_PATH)     # override: A/B runs of another build
    if path == _LIB_PATH and not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(path)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64
    wp = ctypes.POINTER(xfp_weights)
    lib.xfp_gemv.argtypes = [wp, vp, i32, i64, vp, i32, i64, vp]
    lib.xfp_gemv_noalloc.argtypes = [wp, vp, i32, i64, vp, i32, i64, vp]
    lib.xfp_gemv_moe.argtypes = [wp, vp, i32, vp, i64, vp, i32, i64, vp]
    lib.xfp_gemv_moe_silu_mul.argtypes = [wp, vp, i32, vp, i64, vp, i32, i64, vp]
    lib.xfp_unpack_indices.argtypes = [wp, vp, vp]
    lib.xfp_gemv_moe_combine.argtypes = [wp, vp, i32, vp, i64, vp, vp, i32, vp]
    lib.xfp_convert_bf16_to_f16.argtypes = [vp, i64, vp, i32, i32, vp]
    lib.xfp_repack_word10.argtypes = [vp, i64, i32, vp, vp]
    lib.xfp_repack_words.argtypes = [vp, i64, i32, i32, vp, vp]
    lib.xfp_check_contents.argtypes = [wp, i64, vp, i32, vp, vp]
    lib.xfp_dequant_bulk.argtypes = [wp, vp, vp]
    lib.xfp_probe_read.argtypes = [vp, u64, vp, vp]
    lib.xfp_probe_copy.argtypes = [vp, vp, u64, vp]
    lib.xfp_select_kernel.argtypes = [i32]
    lib.xfp_route.argtypes = [wp, i32, i32, ctypes.POINTER(ctypes.c_int)]
    lib.xfp_strerror.argtypes = [i32]
    lib.xfp_strerror.restype = ctypes.c_char_p
    for name in ("xfp_gemv", "xfp_gemv_noalloc", "xfp_gemv_moe", "xfp_gemv_moe_silu_mul", "xfp_gemv_moe_combine", "xfp_check_contents", "xfp_convert_bf16_to_f16", "xfp_repack_word10", "xfp_repack_words", "xfp_unpack_indices", "xfp_dequant_bulk",
                 "xfp_probe_read", "xfp_probe_copy", "xfp_version", "xfp_init", "xfp_select_kernel", "xfp_route"):
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


def xfp_strerror(status: int) -> str:
    return load_library().xfp_strerror(int(status)).decode()


def xfp_version() -> int:
    return int(load_library().xfp_version())


XFP_KERNEL_AUTO, XFP_KERNEL_STREAM, XFP_KERNEL_TILE = 0, 1, 2


def xfp_select_kernel(which: int) -> None:
    """Which kernel M = 1 calls take where two can (measurement and test aid); XFP_KERNEL_AUTO restores the rule."""
    _check(load_library().xfp_select_kernel(int(which)))


XFP_ROUTE_GENERAL, XFP_ROUTE_STREAM, XFP_ROUTE_SPLIT_K, XFP_ROUTE_TILE, XFP_ROUTE_BATCH, XFP_ROUTE_WIDE = range(6)


def xfp_route(W, M: int, expert_indexed: bool = False):
    """(route id, tokens) of the first launch xfp_gemv / xfp_gemv_moe would make for M tokens / slots (host only).
    W: a DeviceWeights or an xfp_weights descriptor."""
    desc = W.desc if hasattr(W, "desc") else W
    n = ctypes.c_int(0)
    r = load_library().xfp_route(ctypes.byref(desc), int(M), int(bool(expert_indexed)), ctypes.byref(n))
    if r < 0:
        _check(r)
    return r, n.value


def xfp_init() -> None:
    """Resolve the library's static device memory on the current device (optional; before graph capture)."""
    _check(load_library().xfp_init())


def _check(status: int):
    if status != 0:
        raise XfpError(status, xfp_strerror(status))


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None or t.numel() == 0:
        return None
    return t.data_ptr()


@dataclass
class DeviceWeights:
    """Device-resident bank plus the host descriptor the C ABI takes."""
    desc: xfp_weights
    tensors: dict = field(default_factory=dict)

    @property
    def N(self): return int(self.desc.N)
    @property
    def K(self): return int(self.desc.K)
    @property
    def E(self): return int(self.desc.E)
    @property
    def bits(self): return int(self.desc.bits)
    @property
    def mode(self): return int(self.desc.mode)


XFP_FLAG_GROUP_AFFINE = 1


def make_descriptor(mode, bits, N, K, L, E, indices, codebooks, group_ids, out_row_ptr, out_col,
                    out_val, group=128, group_scale=None, group_mid=None) -> DeviceWeights:
    """Wrap device tensors (already laid out as include/xfp.h states) in a descriptor."""
    d = xfp_weights()
    d.struct_size = ctypes.sizeof(xfp_weights)
    d.mode, d.bits, d.group, d.N, d.K, d.L, d.E = mode, bits, group, N, K, L, E
    d.flags = XFP_FLAG_GROUP_AFFINE if group_scale is not None else 0
    d.reserved = 0
    d.indices, d.codebooks, d.group_ids = _ptr(indices), _ptr(codebooks), _ptr(group_ids)
    d.out_row_ptr, d.out_col, d.out_val = _ptr(out_row_ptr), _ptr(out_col), _ptr(out_val)
    d.group_scale, d.group_mid = _ptr(group_scale), _ptr(group_mid)
    return DeviceWeights(d, dict(indices=indices, codebooks=codebooks, group_ids=group_ids,
                                 out_row_ptr=out_row_ptr, out_col=out_col, out_val=out_val,
                                 group_scale=group_scale, group_mid=group_mid))


def _to_dev(a: Optional[np.ndarray], device, view=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if view is not None:
        a = a.view(view)
    return torch.from_numpy(a).to(device)


def upload(W, device="cuda") -> DeviceWeights:
    """Copy host arrays (xfp_inputs.XfpHostWeights or format.load_xfp output) to the GPU."""
    return make_descriptor(
        W.mode, W.bits, W.N, W.K, W.L, W.E,
        _to_dev(W.indices, device, np.int32), _to_dev(W.codebooks, device, np.int16),
        _to_dev(W.group_ids, device), _to_dev(W.out_row_ptr, device),
        _to_dev(W.out_col, device), _to_dev(W.out_val, device, np.int16), group=W.group,
        group_scale=_to_dev(getattr(W, "group_scale", None), device, np.int16),
        group_mid=_to_dev(getattr(W, "group_mid", None), device, np.int16))


def _y_code(dtype, x: Optional[torch.Tensor] = None) -> int:
    """dtype argument of the C ABI: the output type, plus the flag for bf16 activations."""
    flag = 0
    if x is not None:
        if x.dtype == torch.bfloat16:
            flag = XFP_X_BF16
        elif x.dtype != torch.float16:
            raise XfpError(-3, "x dtype must be torch.float16 or torch.bfloat16")
    if dtype == torch.float16:
        return XFP_F16 | flag
    if dtype == torch.float32:
        return XFP_F32 | flag
    if dtype == torch.bfloat16:
        return XFP_BF16 | flag
    raise XfpError(-3, "y dtype must be torch.float16, torch.bfloat16 or torch.float32")


def xfp_gemv(W: DeviceWeights, x: torch.Tensor, y: Optional[torch.Tensor] = None,
             y_dtype=torch.float16, stream=None) -> torch.Tensor:
    """y[M, N] = x[M, K] * W_hat^T.  x: fp16 device tensor [M, K] or [K], row stride = ldx."""
    x2 = x if x.dim() == 2 else x.unsqueeze(0)
    M = x2.shape[0]
    if y is None:
        y = torch.empty((M, W.N), dtype=y_dtype, device=x.device)
    y2 = y if y.dim() == 2 else y.unsqueeze(0)
    ldx = x2.stride(0) if M > 1 else max(x2.shape[1], 1)
    ldy = y2.stride(0) if M > 1 else max(y2.shape[1], 1)
    _check(load_library().xfp_gemv(ctypes.byref(W.desc), _ptr(x2), M, ldx, _ptr(y2),
                                   _y_code(y2.dtype, x2), ldy, _stream(stream)))
    return y


def xfp_gemv_noalloc(W: DeviceWeights, x: torch.Tensor, y: torch.Tensor, stream=None) -> torch.Tensor:
    """xfp_gemv with its scratch in the library's one static array; the caller brings y (nothing is allocated)."""
    x2 = x if x.dim() == 2 else x.unsqueeze(0)
    M = x2.shape[0]
    y2 = y if y.dim() == 2 else y.unsqueeze(0)
    ldx = x2.stride(0) if M > 1 else max(x2.shape[1], 1)
    ldy = y2.stride(0) if M > 1 else max(y2.shape[1], 1)
    _check(load_library().xfp_gemv_noalloc(ctypes.byref(W.desc), _ptr(x2), M, ldx, _ptr(y2),
                                           _y_code(y2.dtype, x2), ldy, _stream(stream)))
    return y


def xfp_gemv_moe(bank: DeviceWeights, expert_ids: torch.Tensor, x: torch.Tensor,
                 y: Optional[torch.Tensor] = None, y_dtype=torch.float16, stream=None) -> torch.Tensor:
    """y[t, :] = matrix expert_ids[t] applied to x[t] (x [T, K]) or to the shared x (x [K] or [1, K])."""
    T = int(expert_ids.numel())
    shared = x.dim() == 1 or x.shape[0] == 1 and T != 1
    x_slot_stride = 0 if shared else x.stride(0)
    if y is None:
        y = torch.empty((T, bank.N), dtype=y_dtype, device=x.device)
    ldy = y.stride(0) if y.dim() == 2 and T > 1 else bank.N
    _check(load_library().xfp_gemv_moe(ctypes.byref(bank.desc), _ptr(expert_ids), T, _ptr(x),
                                       x_slot_stride, _ptr(y) if T else y.data_ptr(),
                                       _y_code(y.dtype, x), ldy, _stream(stream)))
    return y


def xfp_gemv_moe_silu_mul(bank: DeviceWeights, expert_ids: Optional[torch.Tensor], x: torch.Tensor,
                          h: Optional[torch.Tensor] = None, h_dtype=torch.float16, stream=None) -> torch.Tensor:
    """h[t, j] = SiLU(y[t, j]) * y[t, N/2 + j] with y as xfp_gemv_moe gives it (gate rows first, then up rows).
    expert_ids None: one matrix (bank.E == 1), slot t is row t of x."""
    T = int(expert_ids.numel()) if expert_ids is not None else (1 if x.dim() == 1 else int(x.shape[0]))
    shared = x.dim() == 1 or x.shape[0] == 1 and T != 1
    x_slot_stride = 0 if shared else x.stride(0)
    if h is None:
        h = torch.empty((T, bank.N // 2), dtype=h_dtype, device=x.device)
    ldh = h.stride(0) if h.dim() == 2 and T > 1 else bank.N // 2
    _check(load_library().xfp_gemv_moe_silu_mul(
        ctypes.byref(bank.desc), _ptr(expert_ids) if expert_ids is not None else None, T, _ptr(x), x_slot_stride,
        _ptr(h) if T else h.data_ptr(), _y_code(h.dtype, x), ldh, _stream(stream)))
    return h


def xfp_gemv_moe_combine(bank: DeviceWeights, expert_ids: torch.Tensor, x: torch.Tensor, slot_weights: torch.Tensor,
                         y: Optional[torch.Tensor] = None, y_dtype=torch.float16, stream=None) -> torch.Tensor:
    """y[n] = sum_t slot_weights[t] * (matrix expert_ids[t] applied to x[t])[n]; slot_weights fp32 [T]."""
    T = int(expert_ids.numel())
    assert slot_weights.dtype == torch.float32 and slot_weights.numel() == T
    shared = x.dim() == 1 or x.shape[0] == 1 and T != 1
    x_slot_stride = 0 if shared else x.stride(0)
    if y is None:
        y = torch.empty((bank.N,), dtype=y_dtype, device=x.device)
    _check(load_library().xfp_gemv_moe_combine(ctypes.byref(bank.desc), _ptr(expert_ids), T, _ptr(x), x_slot_stride,
                                               _ptr(slot_weights), _ptr(y), _y_code(y.dtype, x), _stream(stream)))
    return y


def xfp_check_contents(W: DeviceWeights, expert_ids: Optional[torch.Tensor] = None, stream=None) -> dict:
    """Device-side check of group ids, CSR arrays and expert ids; synchronises and returns the report."""
    report = torch.zeros(4, dtype=torch.int32, device="cuda")
    col = W.tensors.get("out_col")
    cap = 0 if col is None else int(col.numel())
    T = 0 if expert_ids is None else int(expert_ids.numel())
    _check(load_library().xfp_check_contents(ctypes.byref(W.desc), cap, _ptr(expert_ids), T, _ptr(report),
                                             _stream(stream)))
    torch.cuda.synchronize()
    r = [int(v) & 0xFFFFFFFF for v in report.cpu().tolist()]
    kinds = [k for k in range(1, 6) if r[1] >> k & 1]
    return {"violations": r[0], "kinds": kinds, "first_position": None if r[0] == 0 else r[2] | r[3] << 32}


def xfp_convert_bf16_to_f16(src: torch.Tensor, stream=None) -> torch.Tensor:
    """fp16 copy of a bf16 tensor [rows, cols] (or [cols]); exact inside fp16's normal range, saturating beyond."""
    s2 = src if src.dim() == 2 else src.unsqueeze(0)
    rows, cols = int(s2.shape[0]), int(s2.shape[1])
    dst = torch.empty((rows, cols), dtype=torch.float16, device=src.device)
    _check(load_library().xfp_convert_bf16_to_f16(_ptr(s2), s2.stride(0) if rows > 1 else cols, _ptr(dst), rows, cols,
                                                  _stream(stream)))
    return dst if src.dim() == 2 else dst[0]


def xfp_repack_word10(words: torch.Tensor, K: int, stream=None) -> torch.Tensor:
    """Dense 3-bit stream [rows, K*3/32] (int32 tensor) of indices stored ten to a uint32 [rows, ceil(K/10)]
    (paper table 2); a one-time conversion at load."""
    w2 = words.reshape(-1, words.shape[-1]).contiguous()
    rows = int(w2.shape[0])
    if w2.element_size() != 4 or int(w2.shape[1]) != (K + 9) // 10:
        raise XfpError(-2, "words must be 32-bit, [rows, ceil(K/10)]")
    dst = torch.empty((rows, K * 3 // 32), dtype=torch.int32, device=words.device)
    _check(load_library().xfp_repack_word10(_ptr(w2), rows, int(K), _ptr(dst), _stream(stream)))
    return dst.reshape(*words.shape[:-1], K * 3 // 32)


def xfp_repack_words(words: torch.Tensor, K: int, bits: int, stream=None) -> torch.Tensor:
    """Dense stream [rows, K*bits/32] (int32 tensor) of indices stored in a word form of the paper's table 2
    (16 / 10 / 8 / 5 per 32-bit word at 2 / 3 / 4 / 6 bits, 3 per 16-bit word at 5 bits); once at load."""
    per = {2: 16, 3: 10, 4: 8, 5: 3, 6: 5}[bits]
    w2 = words.reshape(-1, words.shape[-1]).contiguous()
    rows = int(w2.shape[0])
    if w2.element_size() != (2 if bits == 5 else 4) or int(w2.shape[1]) != (K + per - 1) // per:
        raise XfpError(-2, "words must be 16-bit (5 bits) or 32-bit, [rows, ceil(K/per)]")
    dst = torch.empty((rows, K * bits // 32), dtype=torch.int32, device=words.device)
    _check(load_library().xfp_repack_words(_ptr(w2), rows, int(K), int(bits), _ptr(dst), _stream(stream)))
    return dst.reshape(*words.shape[:-1], K * bits // 32)


def xfp_unpack_indices(W: DeviceWeights, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((W.E * W.N, W.K), dtype=torch.uint8, device="cuda")
    _check(load_library().xfp_unpack_indices(ctypes.byref(W.desc), _ptr(out), _stream(stream)))
    return out


def xfp_dequant_bulk(W: DeviceWeights, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """fp16 bit patterns of Codebook[Q], returned as an int16 tensor [E*N, K]."""
    if out is None:
        out = torch.empty((W.E * W.N, W.K), dtype=torch.int16, device="cuda")
    _check(load_library().xfp_dequant_bulk(ctypes.byref(W.desc), _ptr(out), _stream(stream)))
    return out


def xfp_probe_read(src: torch.Tensor, sink: torch.Tensor, nbytes: Optional[int] = None, stream=None):
    nbytes = src.numel() * src.element_size() if nbytes is None else nbytes
    _check(load_library().xfp_probe_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)))


def xfp_probe_copy(src: torch.Tensor, dst: torch.Tensor, nbytes: Optional[int] = None, stream=None):
    nbytes = src.numel() * src.element_size() if nbytes is None else nbytes
    _check(load_library().xfp_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)))
