"""The CPU reference encoder (paper section 4) against the paper's printed defaults, the properties its steps
must have, and the decode: what it packs is exactly what the oracle unpacks."""
import numpy as np
import pytest

import oracle
import xfp_encoder as enc
import xfp_inputs as xi
from helpers import np_dense_weight


def student_t(N, K, seed, scale=0.02, nu=4.0):
    return scale * np.random.default_rng(seed).standard_t(nu, size=(N, K))


def test_defaults_are_the_papers():
    # section 4.1: k = 4.0, capped at 2 %; section 4.2: 20 rounds; section 3.4: L = 32;
    # section 4.3: floors 0.96 / 0.93, candidates {2, 3, 4} and {2, 4}, four sampled experts
    assert (enc.OUTLIER_K, enc.OUTLIER_CAP, enc.LLOYD_ROUNDS, enc.LIBRARY_SIZE) == (4.0, 0.02, 20, 32)
    assert (enc.TAU_STRICT, enc.TAU_LAZY) == (0.96, 0.93)
    assert enc.CANDIDATES_V2 == (2, 3, 4) and enc.CANDIDATES_V2A == (2, 4) and enc.MOE_SAMPLE_EXPERTS == 4


def test_outlier_extraction_threshold_and_cap():
    rng = np.random.default_rng(0)
    W = rng.normal(0.0, 1.0, size=(256, 1024))
    mask, mu, sigma = enc.extract_outliers(W)
    assert abs(mu) < 0.01 and abs(sigma - 1) < 0.01
    assert np.array_equal(mask, np.abs(W - mu) > 4.0 * sigma)                  # under the cap: exactly the k-sigma rule
    assert 2e-5 < mask.mean() < 2e-4                                           # a Gaussian has 6.3e-5 beyond 4 sigma
    # heavy tails: more than 2 % qualify at k = 1, the cap keeps exactly 2 %, and they are the largest deviations
    Wt = student_t(128, 1024, 1)
    mask, mu, sigma = enc.extract_outliers(Wt, k=1.0)
    assert int(mask.sum()) == int(0.02 * Wt.size)
    dev = np.abs(Wt - mu)
    assert dev[mask].min() >= dev[~mask].max()
    assert enc.extract_outliers(Wt, k=1.0, cap=0.0)[0].sum() == 0


def test_lloyd_starts_at_quantiles_and_never_gets_worse():
    W = student_t(16, 2048, 2)
    cent0 = enc.lloyd_rows(W, 8, rounds=0)
    srt = np.sort(W, axis=1)
    assert np.array_equal(cent0, srt[:, ((np.arange(8) + 0.5) / 8 * 2048).astype(int)])   # CDF-uniform quantiles
    cent, hist = enc.lloyd_rows(W, 8, rounds=20, return_history=True)
    assert len(hist) == 20 and all(b <= a + 1e-18 for a, b in zip(hist, hist[1:]))         # Lloyd's monotone descent
    assert hist[-1] < 0.7 * hist[0]
    assert np.all(np.diff(cent, axis=1) >= 0)
    # run to convergence, the two steps have a fixed point: every entry is the mean of the values nearest to it
    conv = enc.lloyd_rows(W[:4], 8, rounds=400)
    q = enc.nearest_index(W[:4], conv)
    for n in range(4):
        for j in range(8):
            sel = W[n][q[n] == j]
            assert sel.size and abs(sel.mean() - conv[n, j]) < 1e-9
    # one entry per distinct value reproduces the values exactly
    V = np.tile(np.array([-3.0, -1.0, 2.0, 5.0]), (3, 32))
    assert np.array_equal(enc.lloyd_rows(V, 4), np.tile([-3.0, -1.0, 2.0, 5.0], (3, 1)))


@pytest.mark.parametrize("mode", [xi.MODE_V2, xi.MODE_V2A])
def test_cosine_grows_with_the_width_and_what_is_packed_is_what_decodes(mode):
    W = student_t(48, 1024, 3)
    prev = 0.0
    for bits in ((2, 3, 4, 5) if mode == xi.MODE_V2 else (2, 4)):
        e = (enc.encode_v2 if mode == xi.MODE_V2 else enc.encode_v2a)(W, bits)
        med = float(np.median(e.cosine))
        assert med > prev
        prev = med
        hw = e.weights
        # the oracle's dequantised doubles plus the CSR residual are the encoder's own reconstruction, bit for bit
        _, wd = oracle.dequant_bulk(hw.mode, bits, hw.N, hw.K, hw.indices[0], hw.codebooks[0],
                                    None if hw.group_ids is None else hw.group_ids[0],
                                    group_scale=None if hw.group_scale is None else hw.group_scale[0],
                                    group_mid=None if hw.group_mid is None else hw.group_mid[0])
        _, O = np_dense_weight(hw)
        assert np.array_equal(wd + O, e.reconstruction)
        # outliers: at most the cap, strictly ascending columns per row, and the decoded weight there is w to fp16 rounding
        assert hw.nnz <= 0.02 * W.size
        rows = np.repeat(np.arange(hw.N), np.diff(hw.out_row_ptr))
        assert np.all((np.diff(hw.out_col) > 0) | (np.diff(rows) > 0))
        err = np.abs(e.reconstruction[rows, hw.out_col] - W[rows, hw.out_col])
        assert np.all(err <= 2.0 ** -10 * np.abs(W[rows, hw.out_col] - wd[rows, hw.out_col]) + 1e-12)
    assert prev > 0.99


def test_v2a_library_and_group_records():
    W = student_t(96, 512, 4)
    e = enc.encode_v2a(W, 4)
    hw = e.weights
    assert hw.L == 32 and hw.codebooks.shape == (1, 32, 16) and hw.group_ids.max() < 32
    assert hw.group_scale.shape == hw.group_mid.shape == hw.group_ids.shape == (1, 96, 4)
    assert np.all(hw.group_scale.view(np.float16) > 0)
    lib = hw.codebooks[0].view(np.float16).astype(np.float64)
    assert np.all(np.diff(lib, axis=1) >= 0) and lib.min() >= -1.01 and lib.max() <= 1.01   # normalised space
    # fewer channels than L: the library cannot be larger than what it condenses
    assert enc.encode_v2a(W[:8], 2).weights.L == 8


def test_auto_select_returns_the_first_width_that_reaches_the_floor():
    W = student_t(64, 1024, 1)
    bits_s, e_s, tried_s = enc.auto_select(W)
    bits_l, _, tried_l = enc.auto_select(W, routed_expert=True)
    assert tried_s[bits_s] >= 0.96 and all(tried_s[b] < 0.96 for b in tried_s if b < bits_s)
    assert tried_l[bits_l] >= 0.93 and bits_l <= bits_s                        # the lazy floor never asks for more
    assert list(tried_s) == sorted(tried_s) and e_s.bits == bits_s
    # no candidate reaches the floor: the largest one is returned
    bits_f, e_f, tried_f = enc.auto_select(W, tau_strict=0.99999, tau_lazy=0.5)
    assert bits_f == 4 and e_f.bits == 4 and set(tried_f) == {2, 3, 4}
    # V2a skips 3 bits
    assert set(enc.auto_select(W[:, :256], mode=xi.MODE_V2A, tau_strict=0.99999)[2]) == {2, 4}
    with pytest.raises(AssertionError):
        enc.auto_select(W, tau_strict=0.9, tau_lazy=0.95)


def test_moe_selection_runs_on_four_experts():
    experts = np.stack([student_t(16, 256, 10 + e) for e in range(9)])
    bits, tried = enc.auto_select_moe(experts)
    stacked = np.concatenate([experts[e] for e in (0, 2, 5, 8)], axis=0)        # four experts spread over the bank
    assert (bits, tried) == (enc.auto_select(stacked, routed_expert=True)[0], enc.auto_select(stacked, routed_expert=True)[2])
