"""CPU reference encoder for XFP (paper section 4): outlier extraction, per-channel Lloyd codebooks, LibFit,
cosine-floor auto-selection.  numpy only; it PRODUCES packed matrices (xfp_inputs.XfpHostWeights) that the
decode library and the CPU oracle read, and shares no code with either.

This is an input producer, not part of the decode hot path: it exists so that the kernels can be run on
matrices with the index statistics a real encoder gives (non-uniform histograms, residual outliers,
fitted libraries with a scale and a mid-point per group) instead of uniform random words.  The paper's own
weights are not available; the encoder runs on synthetic matrices.

What follows the paper and what is this module's reading:
  section 4.1  mu, sigma over the whole matrix; |w - mu| > k sigma (k = 4.0) goes to the sparse fp16
               residual, at most 2 % of the weights (the largest deviations when more qualify); the bulk
               holds mu at those positions.  Reading: the residual stores w - C[n, k], the difference to
               what the bulk decodes to there, so that the decoded weight is w up to fp16 rounding
               (eq. 1 is a sum; the paper does not say which of the two the residual holds).
  section 4.2  2^N entries per output channel, started at the CDF-uniform quantiles (i + 1/2) / 2^N of the
               channel's bulk, 20 rounds of nearest-entry assignment and conditional-mean update, stored
               as fp16.
  section 3.4  LibFit: a second Lloyd pass over the channels' codebooks condenses them into L = 32; every
               128-weight group is re-indexed against the closest library codebook, with a scale and a
               mid-point of its own.  Reading: mid = (max + min) / 2 and scale = (max - min) / 2 of the
               group's bulk values (scale 1 for a constant group), the library lives in that normalised
               [-1, 1] space, the second pass runs on the channels' normalised codebooks, and a group
               takes the library codebook with the least squared error on its normalised values.
  section 4.3  algorithm 1: candidate widths in ascending order ({2, 3, 4} for V2, {2, 4} for V2a), the
               first whose MEDIAN per-channel cosine similarity between W and its reconstruction reaches
               the floor (0.96 strict, 0.93 for routed experts) is returned, else the largest.
               MoE layers: the selection runs on 4 concatenated experts.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

import xfp_inputs as xi

# the paper's printed defaults (sections 3.4, 4.1, 4.2, 4.3)
OUTLIER_K = 4.0
OUTLIER_CAP = 0.02
LLOYD_ROUNDS = 20
LIBRARY_SIZE = 32
TAU_STRICT = 0.96
TAU_LAZY = 0.93
CANDIDATES_V2 = (2, 3, 4)
CANDIDATES_V2A = (2, 4)
MOE_SAMPLE_EXPERTS = 4
GROUP = 128


def extract_outliers(W: np.ndarray, k: float = OUTLIER_K, cap: float = OUTLIER_CAP):
    """(mask of extracted positions, mu, sigma).  At most cap * W.size positions: the largest deviations."""
    W = np.asarray(W, dtype=np.float64)
    mu, sigma = float(W.mean()), float(W.std())
    dev = np.abs(W - mu)
    mask = dev > k * sigma
    limit = int(cap * W.size)
    if int(mask.sum()) > limit:
        if limit == 0:
            mask[:] = False
        else:
            thr = np.partition(dev.ravel(), W.size - limit)[W.size - limit]
            mask = dev >= thr
            extra = int(mask.sum()) - limit                     # ties at the threshold: drop the surplus deterministically
            if extra > 0:
                ties = np.flatnonzero((dev == thr).ravel())
                mask.ravel()[ties[:extra]] = False
    return mask, mu, sigma


def lloyd_rows(bulk: np.ndarray, levels: int, rounds: int = LLOYD_ROUNDS, return_history: bool = False):
    """Per-row 1-D Lloyd: quantile start, `rounds` of nearest assignment + conditional mean.
    Returns sorted centroids [N, levels] (float64) and, on request, the mean squared error after every round."""
    bulk = np.asarray(bulk, dtype=np.float64)
    N, K = bulk.shape
    srt = np.sort(bulk, axis=1)
    csum = np.concatenate([np.zeros((N, 1)), np.cumsum(srt, axis=1)], axis=1)
    csq = np.concatenate([np.zeros((N, 1)), np.cumsum(srt * srt, axis=1)], axis=1)
    qpos = ((np.arange(levels) + 0.5) / levels * K).astype(np.int64).clip(0, K - 1)
    cent = srt[:, qpos].copy()
    rows = np.arange(N)[:, None]
    hist = []
    for _ in range(rounds):
        mid = 0.5 * (cent[:, 1:] + cent[:, :-1])
        cut = np.empty((N, levels - 1), dtype=np.int64)
        for n in range(N):                                      # a value equal to a boundary goes to the lower cell
            cut[n] = np.searchsorted(srt[n], mid[n], side="right")
        edges = np.concatenate([np.zeros((N, 1), np.int64), cut, np.full((N, 1), K, np.int64)], axis=1)
        cnt = np.diff(edges, axis=1)
        sums = csum[rows, edges[:, 1:]] - csum[rows, edges[:, :-1]]
        if return_history:
            sq = csq[rows, edges[:, 1:]] - csq[rows, edges[:, :-1]]
            hist.append(float((sq - 2 * cent * sums + cnt * cent * cent).sum() / (N * K)))   # error of this round's assignment
        new = np.where(cnt > 0, sums / np.maximum(cnt, 1), cent)                              # an empty cell keeps its entry
        cent = np.sort(new, axis=1)
    return (cent, hist) if return_history else cent


def nearest_index(values: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """Index of the nearest entry of each row's sorted codebook (ties to the lower entry)."""
    N, K = values.shape
    mid = 0.5 * (codebooks[:, 1:] + codebooks[:, :-1])
    q = np.empty((N, K), dtype=np.uint8)
    for n in range(N):
        q[n] = np.searchsorted(mid[n], values[n], side="left")
    return q


@dataclass
class Encoded:
    """An encoded matrix: the packed form the decode reads plus what the encoder knows about it."""
    weights: xi.XfpHostWeights
    reconstruction: np.ndarray          # float64 [N, K]: what the packed form decodes to (fp16 entries and residuals)
    cosine: np.ndarray                  # per output channel, against the original matrix
    bits: int


def per_channel_cosine(W: np.ndarray, What: np.ndarray) -> np.ndarray:
    num = (W * What).sum(axis=1)
    den = np.sqrt((W * W).sum(axis=1) * (What * What).sum(axis=1))
    return np.where(den > 0, num / np.where(den > 0, den, 1.0), 1.0)


def _csr(mask: np.ndarray, values: np.ndarray):
    r, c = np.nonzero(mask)
    row_ptr = np.zeros(mask.shape[0] + 1, dtype=np.int64)
    np.add.at(row_ptr, r + 1, 1)
    return np.cumsum(row_ptr).astype(np.int32), c.astype(np.int32), values[r, c].astype(np.float16).view(np.uint16)


def encode_v2(W: np.ndarray, bits: int, *, k: float = OUTLIER_K, cap: float = OUTLIER_CAP,
              rounds: int = LLOYD_ROUNDS) -> Encoded:
    """One fp16 codebook of 2^bits entries per output channel (sections 4.1, 4.2)."""
    W = np.asarray(W, dtype=np.float64)
    N, K = W.shape
    assert K % GROUP == 0 and 2 <= bits <= 6
    mask, mu, _ = extract_outliers(W, k, cap)
    bulk = np.where(mask, mu, W)
    cb16 = np.sort(lloyd_rows(bulk, 1 << bits, rounds).astype(np.float16), axis=1)
    cbf = cb16.astype(np.float64)
    q = nearest_index(bulk, cbf)
    C = np.take_along_axis(cbf, q.astype(np.int64), axis=1)
    resid = np.where(mask, W - C, 0.0)
    row_ptr, col, val = _csr(mask, resid)
    What = C + np.where(mask, resid.astype(np.float16).astype(np.float64), 0.0)
    hw = xi.XfpHostWeights(mode=xi.MODE_V2, bits=bits, N=N, K=K, E=1, L=0,
                           indices=xi.pack_bitstream(q, bits).reshape(1, N, K * bits // 32),
                           codebooks=cb16.view(np.uint16).reshape(1, N, 1 << bits), group_ids=None,
                           out_row_ptr=row_ptr, out_col=col, out_val=val,
                           meta={"recipe": "reference-encoder-v2", "mu": mu, "outliers": int(mask.sum())})
    return Encoded(hw, What, per_channel_cosine(W, What), bits)


def libfit(codebooks: np.ndarray, L: int = LIBRARY_SIZE, rounds: int = LLOYD_ROUNDS, seed: int = 0) -> np.ndarray:
    """Second Lloyd pass (vector k-means) over codebooks [n, entries] -> library [L, entries], rows sorted."""
    cbs = np.asarray(codebooks, dtype=np.float64)
    n = cbs.shape[0]
    L = min(L, n)
    order = np.argsort(cbs.mean(axis=1), kind="stable")        # deterministic start: evenly spaced along the sorted means
    lib = cbs[order[((np.arange(L) + 0.5) / L * n).astype(np.int64)]].copy()
    for _ in range(rounds):
        d = ((cbs[:, None, :] - lib[None, :, :]) ** 2).sum(axis=2)
        a = d.argmin(axis=1)
        for l in range(L):
            sel = a == l
            if sel.any():
                lib[l] = cbs[sel].mean(axis=0)
    return np.sort(lib, axis=1)


def encode_v2a(W: np.ndarray, bits: int, *, L: int = LIBRARY_SIZE, k: float = OUTLIER_K, cap: float = OUTLIER_CAP,
               rounds: int = LLOYD_ROUNDS) -> Encoded:
    """A library of L codebooks per layer, one id, scale and mid-point per 128-weight group (section 3.4)."""
    W = np.asarray(W, dtype=np.float64)
    N, K = W.shape
    assert K % GROUP == 0 and 2 <= bits <= 6
    G = K // GROUP
    mask, mu, _ = extract_outliers(W, k, cap)
    bulk = np.where(mask, mu, W)
    g = bulk.reshape(N, G, GROUP)
    hi, lo = g.max(axis=2), g.min(axis=2)
    mid16 = (0.5 * (hi + lo)).astype(np.float16)
    half = 0.5 * (hi - lo)
    scale16 = np.where(half > 0, half, 1.0).astype(np.float16)
    scale16 = np.where(scale16.astype(np.float64) > 0, scale16, np.float16(1.0)).astype(np.float16)   # a range below fp16's smallest
    mid, scale = mid16.astype(np.float64), scale16.astype(np.float64)
    u = ((g - mid[:, :, None]) / scale[:, :, None]).reshape(N, K)          # normalised bulk, about [-1, 1]
    lib16 = libfit(lloyd_rows(u, 1 << bits, rounds), L, rounds).astype(np.float16)
    lib16 = np.sort(lib16, axis=1)
    libf = lib16.astype(np.float64)
    Lr = libf.shape[0]
    ug = u.reshape(N * G, GROUP)
    best_err = np.full(N * G, np.inf)
    ids = np.zeros(N * G, dtype=np.uint8)
    qbest = np.zeros((N * G, GROUP), dtype=np.uint8)
    for l in range(Lr):
        ql = np.searchsorted(0.5 * (libf[l, 1:] + libf[l, :-1]), ug, side="left").astype(np.uint8)
        err = ((ug - libf[l][ql]) ** 2).sum(axis=1)
        better = err < best_err
        best_err = np.where(better, err, best_err)
        ids = np.where(better, np.uint8(l), ids)
        qbest[better] = ql[better]
    ids = ids.reshape(N, G)
    q = qbest.reshape(N, K)
    C = (libf[np.repeat(ids.astype(np.int64), GROUP, axis=1), q.astype(np.int64)]
         * np.repeat(scale, GROUP, axis=1) + np.repeat(mid, GROUP, axis=1))
    resid = np.where(mask, W - C, 0.0)
    row_ptr, col, val = _csr(mask, resid)
    What = C + np.where(mask, resid.astype(np.float16).astype(np.float64), 0.0)
    hw = xi.XfpHostWeights(mode=xi.MODE_V2A, bits=bits, N=N, K=K, E=1, L=Lr,
                           indices=xi.pack_bitstream(q, bits).reshape(1, N, K * bits // 32),
                           codebooks=lib16.view(np.uint16).reshape(1, Lr, 1 << bits), group_ids=ids.reshape(1, N, G),
                           out_row_ptr=row_ptr, out_col=col, out_val=val,
                           meta={"recipe": "reference-encoder-v2a", "mu": mu, "outliers": int(mask.sum())},
                           group_scale=scale16.view(np.uint16).reshape(1, N, G), group_mid=mid16.view(np.uint16).reshape(1, N, G))
    return Encoded(hw, What, per_channel_cosine(W, What), bits)


def auto_select(W: np.ndarray, *, routed_expert: bool = False, mode: int = xi.MODE_V2, candidates=None,
                tau_strict: float = TAU_STRICT, tau_lazy: float = TAU_LAZY, **encoder_args):
    """Algorithm 1: (chosen width, its encoding, {width: median cosine} of every width that was tried)."""
    assert tau_lazy <= tau_strict
    tau = tau_lazy if routed_expert else tau_strict
    cands = tuple(sorted(candidates if candidates is not None else (CANDIDATES_V2 if mode == xi.MODE_V2 else CANDIDATES_V2A)))
    tried, enc = {}, None
    for bits in cands:
        enc = (encode_v2 if mode == xi.MODE_V2 else encode_v2a)(W, bits, **encoder_args)
        tried[bits] = float(np.median(enc.cosine))
        if tried[bits] >= tau:
            return bits, enc, tried
    return cands[-1], enc, tried                                # fallback: the largest candidate


def auto_select_moe(experts: np.ndarray, sample: int = MOE_SAMPLE_EXPERTS, **kw):
    """Routed experts [E, N, K]: the width is chosen on `sample` experts concatenated along the output channels."""
    E = experts.shape[0]
    pick = np.linspace(0, E - 1, num=min(sample, E)).astype(np.int64)
    stacked = np.concatenate([experts[e] for e in pick], axis=0)
    bits, _, tried = auto_select(stacked, routed_expert=True, **kw)
    return bits, tried
