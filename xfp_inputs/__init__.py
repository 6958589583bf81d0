"""Seeded synthetic inputs for the XFP fused decode path.

This module only *produces* inputs: packed index tensors, fp16 codebooks,
V2a group ids, CSR outliers, activations and expert ids, as host numpy
arrays.  It holds none of the decode arithmetic (no unpack, no dequant,
no GEMV); both the CPU oracle's tests and the GPU path's tests/bench take
their inputs from here so that they see identical bytes.

Any bit pattern is a valid packed index tensor, so the bit packer below is
input encoding only: a mistake in it would change which valid input is
produced, not whether either side decodes it correctly.

Workload recipes stand in for the paper's layer shapes and weight
statistics (heavy-tailed attention projections with entries tens of sigma
out, near-Gaussian routed experts, 256 experts per MoE layer; paper
sections 1, 6.2 and appendix B).  They are not the paper's model weights.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

GROUP = 128
BASE_SEED = 20260514

MODE_V2 = 0
MODE_V2A = 1


@dataclass
class XfpHostWeights:
    """One bank of E stacked XFP matrices of identical shape, on the host.

    indices    uint32 [E, N, K*bits/32]  row-major little-endian bitstream
    codebooks  uint16 (fp16 bits)  V2: [E, N, 2**bits]   V2a: [E, L, 2**bits]
    group_ids  uint8  [E, N, K/128] (V2a) or None
    group_scale, group_mid  uint16 (fp16 bits) [E, N, K/128] or None: the per-group scale and
               mid-point of a V2a matrix (paper section 3.4), both or neither
    out_row_ptr int32 [E*N + 1], out_col int32 [nnz], out_val uint16 [nnz]
    """
    mode: int
    bits: int
    N: int
    K: int
    E: int
    L: int
    indices: np.ndarray
    codebooks: np.ndarray
    group_ids: Optional[np.ndarray]
    out_row_ptr: np.ndarray
    out_col: np.ndarray
    out_val: np.ndarray
    group: int = GROUP
    meta: dict = field(default_factory=dict)
    group_scale: Optional[np.ndarray] = None
    group_mid: Optional[np.ndarray] = None

    @property
    def nnz(self) -> int:
        return int(self.out_col.shape[0])

    def algorithmic_bytes(self, M: int = 1, y_bytes: int = 2, experts: int | None = None,
                          shared_x: bool = True) -> int:
        """Bytes one call must move: indices + codebooks + ids + CSR + x + y.

        For a bank (E > 1) `experts` active slots are counted, each with its
        own slice; x is counted once when shared between slots.
        """
        T = 1 if experts is None else experts
        per = (self.N * self.K * self.bits // 8)
        if self.mode == MODE_V2:
            per += self.N * (1 << self.bits) * 2
        else:
            per += self.L * (1 << self.bits) * 2 + self.N * (self.K // self.group) * (5 if self.group_scale is not None else 1)
        nnz_per = self.nnz // self.E
        per += 6 * nnz_per + 4 * (self.N + 1)
        xb = M * self.K * 2
        yb = M * self.N * y_bytes
        if experts is None:
            return per + xb + yb
        return T * (per + yb) + (xb if shared_x else T * xb)


def _f16_bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a.astype(np.float16)).view(np.uint16)


def pack_bitstream(q: np.ndarray, bits: int) -> np.ndarray:
    """Encode indices q [..., K] (values < 2**bits) as a dense bitstream.

    Field k occupies bits [k*bits, (k+1)*bits) of its row's stream; the
    stream is stored as little-endian uint32 words, rows are not padded
    (paper table 2 gives the per-word counts for 2 and 4 bits; the dense
    3-bit stream lets fields cross word boundaries).
    """
    q = np.ascontiguousarray(q, dtype=np.uint8)
    K = q.shape[-1]
    assert (K * bits) % 32 == 0
    lead = q.shape[:-1]
    q2 = q.reshape(-1, K)
    out = np.empty((q2.shape[0], K * bits // 8), dtype=np.uint8)
    step = max(1, (1 << 24) // K)
    shifts = np.arange(bits, dtype=np.uint8)
    for r0 in range(0, q2.shape[0], step):
        blk = q2[r0:r0 + step]
        b = ((blk[:, :, None] >> shifts) & 1).astype(np.uint8).reshape(blk.shape[0], K * bits)
        out[r0:r0 + step] = np.packbits(b, axis=1, bitorder="little")
    return out.view("<u4").reshape(*lead, K * bits // 32)


def pack_word10(q: np.ndarray) -> np.ndarray:
    """Encode 3-bit indices q [..., K] ten to a uint32 (paper table 2): value k in word k // 10 at bit
    3 * (k % 10), the top two bits of every word and the unused tail of a row's last word zero."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    K = q.shape[-1]
    wpr = (K + 9) // 10
    q2 = np.zeros((q.size // K, wpr * 10), dtype=np.uint32)
    q2[:, :K] = q.reshape(-1, K)
    w = np.zeros((q2.shape[0], wpr), dtype=np.uint32)
    for j in range(10):
        w |= q2[:, j::10] << np.uint32(3 * j)
    return w.reshape(*q.shape[:-1], wpr)


def pack_wordform(q: np.ndarray, bits: int) -> np.ndarray:
    """Encode indices q [..., K] in the word forms of the paper's table 2: 16 / 10 / 8 / 5 values per uint32 at
    2 / 3 / 4 / 6 bits, 3 per uint16 at 5 bits; value k in word k // per at bit bits * (k % per), reserve bits and
    the unused tail of a row's last word zero."""
    per = {2: 16, 3: 10, 4: 8, 5: 3, 6: 5}[bits]
    wdt = np.uint16 if bits == 5 else np.uint32
    q = np.ascontiguousarray(q, dtype=np.uint8)
    K = q.shape[-1]
    wpr = (K + per - 1) // per
    q2 = np.zeros((q.size // K, wpr * per), dtype=np.uint32)
    q2[:, :K] = q.reshape(-1, K)
    w = np.zeros((q2.shape[0], wpr), dtype=np.uint32)
    for j in range(per):
        w |= q2[:, j::per] << np.uint32(bits * j)
    return w.astype(wdt).reshape(*q.shape[:-1], wpr)


def random_words(rng: np.random.Generator, shape) -> np.ndarray:
    """Uniform random packed words = uniform random indices for any bit width."""
    return rng.integers(0, 1 << 32, size=shape, dtype=np.uint32)


def sorted_normal_codebooks(rng: np.random.Generator, shape, sigma: float = 0.02) -> np.ndarray:
    """fp16 codebooks whose entries are ascending N(0, sigma) draws (last axis)."""
    cb = np.sort(rng.normal(0.0, sigma, size=shape), axis=-1)
    return _f16_bits(cb)


def random_csr(rng_pos: np.random.Generator, rng_val: np.random.Generator, rows: int, K: int,
               nnz: int, val_sigma: float = 0.5):
    """nnz distinct positions uniform over rows x K, fp16 values val_sigma*N(0,1)."""
    total = rows * K
    if nnz > 0:
        pos = np.sort(rng_pos.choice(total, size=nnz, replace=False).astype(np.int64))
    else:
        pos = np.zeros(0, dtype=np.int64)
    r = pos // K
    col = (pos % K).astype(np.int32)
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    np.add.at(row_ptr, r + 1, 1)
    row_ptr = np.cumsum(row_ptr).astype(np.int32)
    val = _f16_bits(val_sigma * rng_val.normal(size=nnz))
    return row_ptr, col, val


def csr_from_dense_mask(mask: np.ndarray, values: np.ndarray):
    """CSR (int32 row_ptr, int32 col, fp16-bit val) of values[mask], row-major."""
    rows, _ = mask.shape
    r, c = np.nonzero(mask)
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    np.add.at(row_ptr, r + 1, 1)
    return (np.cumsum(row_ptr).astype(np.int32), c.astype(np.int32),
            _f16_bits(values[r, c]))


def activations(rng: np.random.Generator, M: int, K: int) -> np.ndarray:
    """x as fp16 bit patterns [M, K], N(0,1)."""
    return _f16_bits(rng.normal(size=(M, K)))


def _streams(seed: int):
    """Sub-streams in fixed order: indices, codebooks, ids, outlier positions,
    outlier values, x, expert ids."""
    ss = np.random.SeedSequence(seed)
    return [np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(7)]


def random_weights(mode: int, bits: int, N: int, K: int, *, E: int = 1, L: int = 32,
                   density: float = 0.003, seed: int = 0, cb_sigma: float = 0.02,
                   val_sigma: float = 0.5, nnz_per_expert: int | None = None, affine: bool = False) -> XfpHostWeights:
    """Uniform-random indices, sorted-normal codebooks, uniform-random outliers.
    affine (V2a): every group also gets a scale (uniform in [0.5, 2)) and a mid-point (N(0, cb_sigma / 2))."""
    assert K % GROUP == 0 and bits in (2, 3, 4, 5, 6) and not (affine and mode != MODE_V2A)
    r_idx, r_cb, r_id, r_pos, r_val, _, _ = _streams(seed)
    indices = random_words(r_idx, (E, N, K * bits // 32))
    if mode == MODE_V2:
        codebooks = sorted_normal_codebooks(r_cb, (E, N, 1 << bits), cb_sigma)
        ids = None
        Lx = 0
    else:
        codebooks = sorted_normal_codebooks(r_cb, (E, L, 1 << bits), cb_sigma)
        ids = r_id.integers(0, L, size=(E, N, K // GROUP), dtype=np.uint8)
        Lx = L
    if nnz_per_expert is None:
        nnz_per_expert = int(round(density * N * K))
    ptrs, cols, vals = [], [], []
    base = 0
    for _ in range(E):
        rp, c, v = random_csr(r_pos, r_val, N, K, nnz_per_expert, val_sigma)
        ptrs.append(rp[:-1].astype(np.int64) + base)
        base += int(rp[-1])
        cols.append(c)
        vals.append(v)
    row_ptr = np.concatenate(ptrs + [np.array([base], dtype=np.int64)]).astype(np.int32)
    gscale = gmid = None
    if affine:
        r_aff = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 7])))    # a stream of its own
        gscale = _f16_bits(r_aff.uniform(0.5, 2.0, size=(E, N, K // GROUP)))
        gmid = _f16_bits(r_aff.normal(0.0, cb_sigma / 2, size=(E, N, K // GROUP)))
    return XfpHostWeights(mode=mode, bits=bits, N=N, K=K, E=E, L=Lx, indices=indices,
                          codebooks=codebooks, group_ids=ids, out_row_ptr=row_ptr,
                          out_col=np.concatenate(cols) if cols else np.zeros(0, np.int32),
                          out_val=np.concatenate(vals) if vals else np.zeros(0, np.uint16),
                          meta={"recipe": "uniform-random", "seed": seed}, group_scale=gscale, group_mid=gmid)


def _lloyd_rows(bulk: np.ndarray, levels: int, iters: int) -> np.ndarray:
    """Per-row 1-D k-means: CDF-uniform quantile start, `iters` rounds of
    nearest-assign + conditional mean (the encoder of paper section 4.2,
    used here only to give the indices a realistic, non-uniform histogram)."""
    N, K = bulk.shape
    srt = np.sort(bulk, axis=1)
    csum = np.concatenate([np.zeros((N, 1)), np.cumsum(srt, axis=1, dtype=np.float64)], axis=1)
    qpos = ((np.arange(levels) + 0.5) / levels * K).astype(np.int64).clip(0, K - 1)
    cent = srt[:, qpos].astype(np.float64)
    for _ in range(iters):
        mid = 0.5 * (cent[:, 1:] + cent[:, :-1])
        new = cent.copy()
        for n in range(N):
            cut = np.searchsorted(srt[n], mid[n], side="left")
            edges = np.concatenate([[0], cut, [K]])
            cnt = np.diff(edges)
            sums = csum[n, edges[1:]] - csum[n, edges[:-1]]
            ok = cnt > 0
            new[n, ok] = sums[ok] / cnt[ok]
        cent = np.sort(new, axis=1)
    return cent


def student_t_weights(N: int, K: int, *, bits: int = 4, density: float = 0.003, seed: int = 0,
                      nu: float = 4.0, scale: float = 0.02, lloyd_iters: int = 5,
                      plant_rows: int = 16, plant_per_row: int = 2,
                      plant_sigma: float = 49.0) -> XfpHostWeights:
    """V2 matrix fitted to heavy-tailed weights.

    W = scale * Student-t(nu); the top `density` fraction by |w - mu| / sigma
    become fp16 outliers holding w (their bulk position is set to mu, paper
    section 4.1); a block of rows additionally gets entries at plant_sigma
    times the matrix sigma (the 49-sigma projection rows of paper section
    6.2); each row's codebook is a short Lloyd fit of its bulk and the
    indices are the nearest fp16 codebook entry.
    """
    r_idx, r_cb, _, r_pos, r_val, _, _ = _streams(seed)
    W = scale * r_idx.standard_t(nu, size=(N, K))
    mu, sd = float(W.mean()), float(W.std())
    pr0 = (N // 16) if N >= 32 else 0
    plant_rows = min(plant_rows, N - pr0)
    for r in range(pr0, pr0 + plant_rows):
        cols = r_pos.choice(K, size=min(plant_per_row, K), replace=False)
        sign = np.where(r_val.random(cols.shape[0]) < 0.5, -1.0, 1.0)
        W[r, cols] = mu + sign * plant_sigma * sd
    nnz = int(round(density * N * K))
    dev = np.abs(W - mu)
    if nnz > 0:
        thr = np.partition(dev.ravel(), N * K - nnz)[N * K - nnz]
        mask = dev >= thr
    else:
        mask = np.zeros_like(W, dtype=bool)
    row_ptr, col, val = csr_from_dense_mask(mask, W)
    bulk = np.where(mask, mu, W)
    cent = _lloyd_rows(bulk, 1 << bits, lloyd_iters)
    cb16 = np.sort(cent.astype(np.float16), axis=1)
    cbf = cb16.astype(np.float64)
    mid = 0.5 * (cbf[:, 1:] + cbf[:, :-1])
    q = np.empty((N, K), dtype=np.uint8)
    for n in range(N):
        q[n] = np.searchsorted(mid[n], bulk[n], side="left")
    indices = pack_bitstream(q, bits).reshape(1, N, K * bits // 32)
    return XfpHostWeights(mode=MODE_V2, bits=bits, N=N, K=K, E=1, L=0, indices=indices,
                          codebooks=cb16.view(np.uint16).reshape(1, N, 1 << bits), group_ids=None,
                          out_row_ptr=row_ptr, out_col=col, out_val=val,
                          meta={"recipe": "student-t-lloyd", "seed": seed, "mu": mu, "sigma": sd,
                                "planted_rows": (pr0, pr0 + plant_rows)})


# ---------------------------------------------------------------------------
# The five measured workloads.  `scale_down` shrinks N (and E) for tests while
# keeping K, bit width, mode, densities and value distributions.
# ---------------------------------------------------------------------------

CONFIG_NAMES = {
    1: "C1 V2 512x1024 b4 M=1",
    2: "C2 V2 8192x4096 b4 M=1 (Student-t fit)",
    3: "C3 V2a 4096x4096 b3 L=32 M=1",
    4: "C4 MoE 8-of-256, gate_up 2048x4096 + down 4096x1024, V2 b3",
    5: "C5 V2 28672x8192 b4 M=16",
}


def config_x(i: int, M: int, K: int, seed: int | None = None) -> np.ndarray:
    seed = BASE_SEED + i if seed is None else seed
    return activations(_streams(seed)[5], M, K)


def config_weights(i: int, *, seed: int | None = None, N: int | None = None,
                   E: int | None = None):
    """Weights of workload i (1..5).  Workload 4 returns (gate_up, down)."""
    seed = BASE_SEED + i if seed is None else seed
    if i == 1:
        return random_weights(MODE_V2, 4, N or 512, 1024, density=0.003, seed=seed)
    if i == 2:
        return student_t_weights(N or 8192, 4096, bits=4, density=0.003, seed=seed)
    if i == 3:
        return random_weights(MODE_V2A, 3, N or 4096, 4096, L=32, density=0.001, seed=seed)
    if i == 4:
        E = 256 if E is None else E
        gu = random_weights(MODE_V2, 3, N or 2048, 4096, E=E, density=0.0005, seed=seed)
        dn = random_weights(MODE_V2, 3, (2 * N) if N else 4096, 1024, E=E, density=0.0005,
                            seed=seed + 1000)
        return gu, dn
    if i == 5:
        return random_weights(MODE_V2, 4, N or 28672, 8192, density=0.003, seed=seed)
    raise ValueError(f"no workload {i}")


def config_expert_ids(i: int, T: int, E: int, seed: int | None = None, draw: int = 0) -> np.ndarray:
    """T distinct expert ids in [0, E); `draw` selects successive routings."""
    seed = BASE_SEED + i if seed is None else seed
    rng = _streams(seed)[6]
    out = None
    for _ in range(draw + 1):
        out = rng.choice(E, size=T, replace=False).astype(np.int32)
    return out
