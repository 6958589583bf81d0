"""Shared test helpers: error metric and an independent numpy formulation."""
import numpy as np


def gated_rel_err(y_hat, y_ref):
    """max |y_hat - y| / max(|y|, 0.01 * rms(y)): element-wise relative error
    with a floor, because y is a zero-mean sum and some |y[n]| are tiny."""
    y_hat = np.asarray(y_hat, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    rms = np.sqrt(np.mean(y_ref ** 2)) if y_ref.size else 0.0
    den = np.maximum(np.abs(y_ref), max(0.01 * rms, 1e-30))
    return float(np.max(np.abs(y_hat - y_ref) / den)) if y_ref.size else 0.0


def np_unpack(words, K, bits):
    """Independent unpack: numpy bit expansion (not the oracle's loop)."""
    w = np.ascontiguousarray(words, dtype="<u4")
    rows = w.size // (K * bits // 32)
    b = np.unpackbits(w.reshape(rows, -1).view(np.uint8), axis=1, bitorder="little")
    b = b.reshape(rows, K, bits).astype(np.uint32)
    return (b << np.arange(bits, dtype=np.uint32)).sum(axis=2).astype(np.uint8)


def bigint_pack(q_row, bits):
    """Independent pack of one row through Python big-integer arithmetic."""
    big = 0
    for k, v in enumerate(q_row):
        big |= int(v) << (k * bits)
    nwords = len(q_row) * bits // 32
    return np.array([(big >> (32 * i)) & 0xFFFFFFFF for i in range(nwords)], dtype=np.uint32)


def np_dense_weight(W, e=0):
    """Dense fp64 W_hat = Codebook[Q] + W_outlier of matrix e by numpy fancy indexing."""
    q = np_unpack(W.indices[e], W.K, W.bits).astype(np.int64)
    cb = W.codebooks[e].view(np.float16).astype(np.float64)
    if W.mode == 0:
        C = np.take_along_axis(cb, q, axis=1)
    else:
        ids = np.repeat(W.group_ids[e].astype(np.int64), W.group, axis=1)
        C = cb[ids, q]
    O = np.zeros((W.N, W.K))
    rp = W.out_row_ptr[e * W.N:(e + 1) * W.N + 1].astype(np.int64)
    rows = np.repeat(np.arange(W.N), np.diff(rp))
    sl = slice(rp[0], rp[-1])
    O[rows, W.out_col[sl]] = W.out_val[sl].view(np.float16).astype(np.float64)
    return C, O


def np_gemv(W, x_bits, e=0):
    C, O = np_dense_weight(W, e)
    x = np.asarray(x_bits, dtype=np.uint16).reshape(-1, W.K).view(np.float16).astype(np.float64)
    return x @ (C + O).T
