"""ctypes front end of the C oracle (xfp_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It never touches the GPU and shares nothing with the HIP
library; numpy arrays in, numpy arrays out.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "xfp_oracle.c")
_LIB = os.path.join(_HERE, "libxfp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.xfp_oracle_max_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def max_threads() -> int:
    return int(_load().xfp_oracle_max_threads())


def half_to_double(h: np.ndarray) -> np.ndarray:
    h = _c(h, np.uint16)
    out = np.empty(h.shape, dtype=np.float64)
    _load().xfp_oracle_half_to_double(_p(h), ctypes.c_int64(h.size), _p(out))
    return out


def unpack(words: np.ndarray, K: int, bits: int) -> np.ndarray:
    """words uint32 [..., K*bits/32] -> indices uint8 [..., K]."""
    words = _c(words, np.uint32)
    rows = words.size // (K * bits // 32)
    q = np.empty((rows, K), dtype=np.uint8)
    _load().xfp_oracle_unpack(_p(words), ctypes.c_int64(rows), ctypes.c_int64(K),
                              ctypes.c_int(bits), _p(q))
    return q.reshape(*words.shape[:-1], K)


def pack(q: np.ndarray, bits: int) -> np.ndarray:
    q = _c(q, np.uint8)
    K = q.shape[-1]
    rows = q.size // K
    words = np.empty((rows, K * bits // 32), dtype=np.uint32)
    _load().xfp_oracle_pack(_p(q), ctypes.c_int64(rows), ctypes.c_int64(K), ctypes.c_int(bits),
                            _p(words))
    return words.reshape(*q.shape[:-1], K * bits // 32)


def unpack_word10(words: np.ndarray, K: int) -> np.ndarray:
    """3-bit indices in the ten-per-uint32 packing (paper table 2): words [..., ceil(K/10)] -> uint8 [..., K]."""
    words = _c(words, np.uint32)
    wpr = (K + 9) // 10
    rows = words.size // wpr
    q = np.empty((rows, K), dtype=np.uint8)
    _load().xfp_oracle_unpack_word10(_p(words), ctypes.c_int64(rows), ctypes.c_int64(K), _p(q))
    return q.reshape(*words.shape[:-1], K)


def repack_word10(words: np.ndarray, K: int) -> np.ndarray:
    """The same indices as the dense 3-bit stream: unpack every value, pack it again."""
    return pack(unpack_word10(words, K), 3)


def unpack_wordform(words: np.ndarray, K: int, bits: int) -> np.ndarray:
    """Indices stored in the word forms of the paper's table 2 (2: 16 per uint32, 3: 10 per uint32, 4: 8 per
    uint32, 5: 3 per uint16, 6: 5 per uint32; reserve bits ignored): words [..., ceil(K/per)] -> uint8 [..., K]."""
    per = {2: 16, 3: 10, 4: 8, 5: 3, 6: 5}[bits]
    wdt = np.uint16 if bits == 5 else np.uint32
    words = _c(words, wdt)
    wpr = (K + per - 1) // per
    rows = words.size // wpr
    q = np.empty((rows, K), dtype=np.uint8)
    raw = np.ascontiguousarray(words).view(np.uint8)
    got = _load().xfp_oracle_unpack_wordform(_p(raw), ctypes.c_int64(rows), ctypes.c_int64(K), ctypes.c_int(bits), _p(q))
    assert got == per
    return q.reshape(*words.shape[:-1], K)


def repack_wordform(words: np.ndarray, K: int, bits: int) -> np.ndarray:
    """The same indices as the dense stream: unpack every value, pack it again."""
    return pack(unpack_wordform(words, K, bits), bits)


def dequant_bulk(mode, bits, N, K, words, codebooks, group_ids=None, want_double=True, group_scale=None, group_mid=None):
    """Bulk term of one matrix: (fp16 bit patterns of the selected entries [N,K], bulk values as doubles or None;
    the doubles include the per-group scale and mid-point when given)."""
    words, codebooks = _c(words, np.uint32), _c(codebooks, np.uint16)
    group_ids = _c(group_ids, np.uint8)
    group_scale, group_mid = _c(group_scale, np.uint16), _c(group_mid, np.uint16)
    wb = np.empty((N, K), dtype=np.uint16)
    wd = np.empty((N, K), dtype=np.float64) if want_double else None
    rc = _load().xfp_oracle_dequant_bulk(ctypes.c_int(mode), ctypes.c_int(bits), ctypes.c_int64(N),
                                         ctypes.c_int64(K), _p(words), _p(codebooks),
                                         _p(group_ids), _p(group_scale), _p(group_mid), _p(wb), _p(wd))
    if rc:
        raise ValueError(f"oracle dequant_bulk rejected arguments ({rc})")
    return wb, wd


def gemv(mode, bits, N, K, words, codebooks, group_ids, row_ptr, col, val, x, threads=None, group_scale=None, group_mid=None):
    """y double [M,N] for one matrix; x is fp16 bits [M,K] (or [K])."""
    x = _c(x, np.uint16)
    x2 = x.reshape(-1, K)
    M = x2.shape[0]
    y = np.empty((M, N), dtype=np.float64)
    words, codebooks = _c(words, np.uint32), _c(codebooks, np.uint16)
    group_ids = _c(group_ids, np.uint8)
    row_ptr, col, val = _c(row_ptr, np.int32), _c(col, np.int32), _c(val, np.uint16)
    group_scale, group_mid = _c(group_scale, np.uint16), _c(group_mid, np.uint16)
    rc = _load().xfp_oracle_gemv(ctypes.c_int(mode), ctypes.c_int(bits), ctypes.c_int64(N),
                                 ctypes.c_int64(K), _p(words), _p(codebooks), _p(group_ids),
                                 _p(group_scale), _p(group_mid), _p(row_ptr), _p(col), _p(val), _p(x2), ctypes.c_int64(M),
                                 ctypes.c_int64(K), _p(y), ctypes.c_int64(N),
                                 ctypes.c_int(threads or max_threads()))
    if rc:
        raise ValueError(f"oracle gemv rejected arguments ({rc})")
    return y


def gemv_weights(W, x, threads=None):
    """gemv on an xfp_inputs.XfpHostWeights holding a single matrix (E == 1)."""
    assert W.E == 1
    return gemv(W.mode, W.bits, W.N, W.K, W.indices[0], W.codebooks[0],
                None if W.group_ids is None else W.group_ids[0],
                W.out_row_ptr, W.out_col, W.out_val, x, threads,
                None if getattr(W, "group_scale", None) is None else W.group_scale[0],
                None if getattr(W, "group_mid", None) is None else W.group_mid[0])


def gemv_moe(W, expert_ids, x, shared_x: bool, threads=None):
    """y double [T,N]: slot t = matrix expert_ids[t] applied to x[t] (or the shared x)."""
    ids = _c(expert_ids, np.int32)
    T = ids.shape[0]
    x = _c(x, np.uint16).reshape(-1, W.K)
    stride = 0 if shared_x else W.K
    assert x.shape[0] == (1 if shared_x else T)
    y = np.empty((T, W.N), dtype=np.float64)
    words, codebooks = _c(W.indices, np.uint32), _c(W.codebooks, np.uint16)
    gids = _c(W.group_ids, np.uint8)
    gs, gm = _c(getattr(W, "group_scale", None), np.uint16), _c(getattr(W, "group_mid", None), np.uint16)
    rc = _load().xfp_oracle_gemv_moe(
        ctypes.c_int(W.mode), ctypes.c_int(W.bits), ctypes.c_int64(W.N), ctypes.c_int64(W.K),
        ctypes.c_int64(W.L), ctypes.c_int64(W.E), _p(words), _p(codebooks), _p(gids), _p(gs), _p(gm),
        _p(_c(W.out_row_ptr, np.int32)), _p(_c(W.out_col, np.int32)), _p(_c(W.out_val, np.uint16)),
        _p(ids), ctypes.c_int64(T), _p(x), ctypes.c_int64(stride), _p(y), ctypes.c_int64(W.N),
        ctypes.c_int(threads or max_threads()))
    if rc:
        raise ValueError(f"oracle gemv_moe rejected arguments ({rc})")
    return y


def silu_mul(y: np.ndarray) -> np.ndarray:
    """h[..., j] = SiLU(y[..., j]) * y[..., N/2 + j] in double, SiLU(g) = g / (1 + exp(-g)): the activation of a
    gated-MLP expert (the paper's models, section 6.1, are mixtures of such experts; the paper does not print
    the formula, this is the standard one) applied to a gate/up projection whose gate rows come first."""
    y = np.asarray(y, dtype=np.float64)
    half = y.shape[-1] // 2
    assert y.shape[-1] == 2 * half
    g, u = y[..., :half], y[..., half:]
    with np.errstate(over="ignore"):
        return g / (1.0 + np.exp(-g)) * u


def moe_combine(y: np.ndarray, slot_weights: np.ndarray) -> np.ndarray:
    """out[n] = sum_t slot_weights[t] * y[t, n] in double: the router's weighted sum over the active experts'
    outputs (the paper's models are top-k routed mixtures of experts, section 6.1; the paper does not print the
    formula, this is the standard one).  slot_weights are taken as given (fp32 values, widened exactly)."""
    y = np.asarray(y, dtype=np.float64)
    w = np.asarray(slot_weights, dtype=np.float32).astype(np.float64)
    assert y.ndim == 2 and w.shape == (y.shape[0],)
    out = np.zeros(y.shape[1], dtype=np.float64)
    for t in range(y.shape[0]):
        out += w[t] * y[t]
    return out
