"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these re-use the oracle's own formulas: expected values come from
hand-written bit patterns, Python big-integer arithmetic, numpy's own fp16
converter and bit expansion, closed forms (row sums), dense scatter + numpy
matmul, and textbook symmetric int4 dequantisation.
"""
import math
import os

import numpy as np
import pytest

import oracle
import xfp_inputs as xi
from helpers import bigint_pack, gated_rel_err, np_dense_weight, np_gemv, np_unpack

V2, V2A = xi.MODE_V2, xi.MODE_V2A
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_size_facts.txt")


def f16(a):
    return np.asarray(a, dtype=np.float16).view(np.uint16)


# ------------------------------------------------------------------ fp16 widening
def test_half_to_double_all_patterns():
    h = np.arange(65536, dtype=np.uint16)
    got = oracle.half_to_double(h)
    ref = h.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))   # -0.0 keeps its sign


# ------------------------------------------------------------------ pack / unpack
def test_unpack_hand_vector_3bit_straddle():
    # field 0 = 7 -> bits 0..2 of word 0; field 10 = 5 = 0b101 -> bits 30, 31 of
    # word 0 and bit 0 of word 1 (bit 30 = 1, bit 31 = 0, bit 32 = 1).
    words = np.array([[0x40000007, 0x00000001, 0x00000000]], dtype=np.uint32)
    q = oracle.unpack(words, 32, 3)
    exp = np.zeros((1, 32), dtype=np.uint8)
    exp[0, 0], exp[0, 10] = 7, 5
    assert np.array_equal(q, exp)
    assert np.array_equal(oracle.pack(exp, 3), words)
    # field 21 = 6 = 0b110 -> bits 63 (word 1 bit 31), 64, 65 (word 2 bits 0, 1)
    words = np.array([[0, 0x00000000, 0x00000003]], dtype=np.uint32)
    exp = np.zeros((1, 32), dtype=np.uint8)
    exp[0, 21] = 6
    assert np.array_equal(oracle.unpack(words, 32, 3), exp)


def test_unpack_hand_vectors_2_and_4_bit():
    # 4-bit: 0x76543210 holds values 0..7 with value 0 in the low bits
    assert oracle.unpack(np.array([[0x76543210]], np.uint32), 8, 4).tolist() == [list(range(8))]
    # 2-bit: 0xE4 = 0b11100100 -> 0,1,2,3
    q = oracle.unpack(np.array([[0x000000E4]], np.uint32), 16, 2)
    assert q[0, :4].tolist() == [0, 1, 2, 3] and not q[0, 4:].any()


def test_values_per_word_match_paper_table():
    facts = {}
    for line in open(GOLDEN):
        t = line.split("#")[0].split()
        if t and t[0] == "pack":
            facts[int(t[1])] = tuple(int(v) for v in t[2:])
    for bits in (2, 4):                      # zero reserve bits: dense stream == word packing
        vals, word, used, reserve = facts[bits]
        assert reserve == 0 and used == word == 32 and vals * bits == 32
        q = np.arange(vals, dtype=np.uint8).reshape(1, -1) % (1 << bits)
        w = oracle.pack(q, bits)
        assert w.shape == (1, 1)
        assert int(w[0, 0]) == sum(int(v) << (bits * i) for i, v in enumerate(q[0]))
    assert facts[3] == (10, 32, 30, 2)       # the paper's own 3-bit word form is a different layout


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("K", [128, 384, 1024, 8192])
def test_pack_unpack_round_trip(bits, K):
    rng = np.random.default_rng(100 * bits + K)
    q = rng.integers(0, 1 << bits, size=(5, K), dtype=np.uint8)
    w = oracle.pack(q, bits)
    assert w.dtype == np.uint32 and w.shape == (5, K * bits // 32)
    assert np.array_equal(oracle.unpack(w, K, bits), q)
    assert np.array_equal(w[0], bigint_pack(q[0], bits))          # independent encoder
    assert np.array_equal(xi.pack_bitstream(q, bits), w)          # the generators' encoder
    assert np.array_equal(np_unpack(w, K, bits), q)               # independent decoder
    words = rng.integers(0, 1 << 32, size=(3, K * bits // 32), dtype=np.uint32)
    assert np.array_equal(oracle.pack(oracle.unpack(words, K, bits), bits), words)


# ten 3-bit values per uint32 (paper table 2: 30 bits used, 2 reserved)
def test_word10_hand_vector_and_reserved_bits():
    vals, word, used, reserve = 10, 32, 30, 2
    assert vals * 3 == used and used + reserve == word
    # octal digits are 3-bit fields: 0o1076543210 holds values 0..7, 0, 1 with value 0 in the low bits
    w = np.array([[0o1076543210, 0o0000000052]], dtype=np.uint32)
    q = oracle.unpack_word10(w, 12)
    assert q.tolist() == [[0, 1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 5]]
    w_res = w | np.uint32(0xC0000000)                                 # the reserved bits carry nothing
    assert np.array_equal(oracle.unpack_word10(w_res, 12), q)
    # a row of K values takes ceil(K / 10) words: 128 values -> 13 words, the last holds 8
    q = (np.arange(256, dtype=np.uint8) * 5 % 8).reshape(2, 128)
    w = xi.pack_word10(q)
    assert w.shape == (2, 13) and not (w >> np.uint32(30)).any() and not (w[:, 12] >> np.uint32(24)).any()
    assert np.array_equal(oracle.unpack_word10(w, 128), q)
    assert int(w[1, 3]) == sum(int(q[1, 30 + j]) << (3 * j) for j in range(10))


@pytest.mark.parametrize("K", [128, 384, 4096])
def test_word10_repack_is_the_dense_stream_of_the_same_indices(K):
    rng = np.random.default_rng(K)
    q = rng.integers(0, 8, size=(7, K), dtype=np.uint8)
    w10 = xi.pack_word10(q)
    dense = oracle.repack_word10(w10, K)
    assert dense.shape == (7, K * 3 // 32)
    assert np.array_equal(dense, xi.pack_bitstream(q, 3))             # the generators' dense encoder
    assert np.array_equal(dense[0], bigint_pack(q[0], 3))             # independent encoder
    assert np.array_equal(np_unpack(dense, K, 3), q)                  # independent decoder
    junk = rng.integers(0, 4, size=w10.shape, dtype=np.uint32) << np.uint32(30)
    assert np.array_equal(oracle.repack_word10(w10 | junk, K), dense)


# ------------------------------------------------------------------ bulk term
@pytest.mark.parametrize("mode,bits", [(V2, 2), (V2, 3), (V2, 4), (V2A, 3), (V2A, 4)])
def test_all_ones_codebooks_give_row_sums(mode, bits):
    W = xi.random_weights(mode, bits, 24, 512, density=0.01, seed=7)
    W.codebooks[:] = f16(1.0)
    x = xi.activations(np.random.default_rng(3), 2, 512)
    xd = x.view(np.float16).astype(np.float64)
    valsd = W.out_val.view(np.float16).astype(np.float64)
    y = oracle.gemv_weights(W, x)
    for m in range(2):
        s = math.fsum(xd[m])
        for n in range(W.N):
            j0, j1 = W.out_row_ptr[n], W.out_row_ptr[n + 1]
            exp = s + math.fsum(valsd[j0:j1] * xd[m, W.out_col[j0:j1]])
            assert abs(y[m, n] - exp) <= 1e-12 * max(1.0, abs(exp))


def test_uniform_grid_codebook_is_textbook_int4():
    N, K, s = 16, 256, 0.0625
    W = xi.random_weights(V2, 4, N, K, density=0.0, seed=11)
    W.codebooks[0, :, :] = f16((np.arange(16) - 8) * s)
    x = xi.activations(np.random.default_rng(5), 1, K)
    q = np_unpack(W.indices[0], K, 4).astype(np.float64)
    exp = x.view(np.float16).astype(np.float64) @ ((q - 8.0) * s).T
    assert np.allclose(oracle.gemv_weights(W, x), exp, rtol=1e-13, atol=1e-13)


def test_v2a_single_id_equals_v2_shared_codebook():
    N, K, bits, g = 12, 384, 3, 19
    A = xi.random_weights(V2A, bits, N, K, density=0.004, seed=21)
    A.group_ids[:] = g
    B = xi.random_weights(V2, bits, N, K, density=0.004, seed=21)
    B.indices[:] = A.indices
    B.codebooks[0, :, :] = A.codebooks[0, g]
    x = xi.activations(np.random.default_rng(8), 3, K)
    assert np.array_equal(oracle.gemv_weights(A, x), oracle.gemv_weights(B, x))
    wa, _ = oracle.dequant_bulk(V2A, bits, N, K, A.indices[0], A.codebooks[0], A.group_ids[0])
    wb, _ = oracle.dequant_bulk(V2, bits, N, K, B.indices[0], B.codebooks[0])
    assert np.array_equal(wa, wb)


def test_v2a_group_axis_is_k():
    # ids differ per 128-wide group along K: a one-hot x picks a single group.
    N, K, bits = 4, 512, 4
    W = xi.random_weights(V2A, bits, N, K, density=0.0, seed=33)
    q = np_unpack(W.indices[0], K, bits)
    for k in (0, 127, 128, 300, 511):
        x = np.zeros((1, K), dtype=np.float16)
        x[0, k] = 1.0
        y = oracle.gemv_weights(W, x.view(np.uint16))
        for n in range(N):
            cb = W.codebooks[0, W.group_ids[0, n, k // 128]].view(np.float16)
            assert y[0, n] == float(cb[q[n, k]])


@pytest.mark.parametrize("mode,bits", [(V2, 3), (V2, 4), (V2A, 3)])
def test_entry_permutation_relabel_leaves_weights_bit_identical(mode, bits):
    N, K = 8, 256
    W = xi.random_weights(mode, bits, N, K, density=0.0, seed=40 + bits)
    ids = None if W.group_ids is None else W.group_ids[0]
    w0, _ = oracle.dequant_bulk(mode, bits, N, K, W.indices[0], W.codebooks[0], ids)
    rng = np.random.default_rng(1)
    perm = rng.permutation(1 << bits)            # new entry j holds old entry perm[j]
    inv = np.argsort(perm)
    cb2 = W.codebooks[0][:, perm]
    q2 = inv[np_unpack(W.indices[0], K, bits)].astype(np.uint8)
    w1, _ = oracle.dequant_bulk(mode, bits, N, K, xi.pack_bitstream(q2, bits), cb2, ids)
    assert np.array_equal(w0, w1)


def test_dequant_preserves_fp16_bit_patterns_including_subnormals():
    N, K = 2, 128
    W = xi.random_weights(V2, 4, N, K, density=0.0, seed=50)
    W.codebooks[0, 0, :] = np.array([0x0001, 0x8001, 0x03FF, 0x0400, 0x8000, 0x0000, 0x7BFF, 0xFBFF,
                                     0x3C00, 0xBC00, 0x0002, 0x8002, 0x1234, 0x9234, 0x5555, 0xAAAA],
                                    dtype=np.uint16)
    wb, wd = oracle.dequant_bulk(V2, 4, N, K, W.indices[0], W.codebooks[0])
    q = np_unpack(W.indices[0], K, 4)
    assert np.array_equal(wb[0], W.codebooks[0, 0][q[0]])
    assert np.array_equal(wd[0], W.codebooks[0, 0][q[0]].view(np.float16).astype(np.float64))


# ------------------------------------------------------------------ outlier term
def test_zero_codebooks_isolate_outlier_term():
    N, K = 40, 384
    W = xi.random_weights(V2, 3, N, K, density=0.02, seed=60)
    W.codebooks[:] = 0
    x = xi.activations(np.random.default_rng(6), 2, K)
    _, O = np_dense_weight(W)
    exp = x.view(np.float16).astype(np.float64) @ O.T
    assert np.allclose(oracle.gemv_weights(W, x), exp, rtol=1e-13, atol=1e-14)


def test_no_outliers_and_one_row_holding_all():
    N, K = 6, 256
    W = xi.random_weights(V2, 4, N, K, density=0.0, seed=61)
    x = xi.activations(np.random.default_rng(2), 1, K)
    assert W.nnz == 0
    assert np.allclose(oracle.gemv_weights(W, x), np_gemv(W, x), rtol=1e-12, atol=1e-13)
    # every position of row 3 is an outlier, other rows have none
    W.out_row_ptr = np.array([0, 0, 0, 0, K, K, K], dtype=np.int32)
    W.out_col = np.arange(K, dtype=np.int32)
    W.out_val = f16(np.random.default_rng(9).normal(size=K))
    assert np.allclose(oracle.gemv_weights(W, x), np_gemv(W, x), rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ whole y
@pytest.mark.parametrize("mode,bits,N,K", [(V2, 2, 8, 128), (V2, 3, 16, 256), (V2, 4, 16, 512),
                                           (V2A, 3, 7, 384), (V2A, 4, 16, 256), (V2A, 2, 5, 128)])
def test_brute_force_dense_matmul_tiny(mode, bits, N, K):
    W = xi.random_weights(mode, bits, N, K, density=0.02, seed=70 + bits + N)
    x = xi.activations(np.random.default_rng(4), 3, K)
    assert np.allclose(oracle.gemv_weights(W, x), np_gemv(W, x), rtol=1e-12, atol=1e-14)


def test_brute_force_workload_1_in_full():
    W = xi.config_weights(1)
    x = xi.config_x(1, 1, W.K)
    assert (W.N, W.K, W.bits, W.nnz) == (512, 1024, 4, 1573)
    y = oracle.gemv_weights(W, x)
    assert gated_rel_err(y, np_gemv(W, x)) < 1e-11


def test_student_t_recipe_small_against_brute_force():
    W = xi.config_weights(2, N=64)
    x = xi.config_x(2, 1, W.K)
    y = oracle.gemv_weights(W, x)
    assert gated_rel_err(y, np_gemv(W, x)) < 1e-11
    vals = np.abs(W.out_val.view(np.float16).astype(np.float64))
    assert vals.max() > 40 * W.meta["sigma"]          # planted far-out entries are present


def test_linearity_in_x():
    W = xi.random_weights(V2, 4, 10, 256, density=0.01, seed=80)
    rng = np.random.default_rng(12)
    x1 = (rng.integers(-64, 64, size=(1, 256)) / 16.0).astype(np.float16)
    x2 = (rng.integers(-64, 64, size=(1, 256)) / 16.0).astype(np.float16)
    xs = (x1.astype(np.float64) + x2.astype(np.float64)).astype(np.float16)   # exact in fp16
    assert np.array_equal(xs.astype(np.float64), x1.astype(np.float64) + x2.astype(np.float64))
    ys = oracle.gemv_weights(W, xs.view(np.uint16))
    y12 = oracle.gemv_weights(W, x1.view(np.uint16)) + oracle.gemv_weights(W, x2.view(np.uint16))
    assert np.allclose(ys, y12, rtol=1e-12, atol=1e-14)


def test_batched_rows_equal_single_calls_and_threads_do_not_matter():
    W = xi.random_weights(V2, 4, 20, 256, density=0.01, seed=81)
    x = xi.activations(np.random.default_rng(13), 16, 256)
    y = oracle.gemv_weights(W, x, threads=4)
    for m in range(16):
        assert np.array_equal(y[m], oracle.gemv_weights(W, x[m], threads=1)[0])


@pytest.mark.parametrize("mode", [V2, V2A])
def test_moe_slot_equals_single_matrix_call(mode):
    E, N, K, bits = 6, 12, 256, 3
    W = xi.random_weights(mode, bits, N, K, E=E, density=0.01, seed=90)
    ids = np.array([4, 0, 4, 5], dtype=np.int32)                  # duplicates are legal
    xs = xi.activations(np.random.default_rng(14), 1, K)
    xt = xi.activations(np.random.default_rng(15), 4, K)
    y_shared = oracle.gemv_moe(W, ids, xs, shared_x=True)
    y_slot = oracle.gemv_moe(W, ids, xt, shared_x=False)
    for t, e in enumerate(ids):
        assert np.allclose(y_shared[t], np_gemv(W, xs, e)[0], rtol=1e-12, atol=1e-14)
        assert np.allclose(y_slot[t], np_gemv(W, xt[t], e)[0], rtol=1e-12, atol=1e-14)
        rp = W.out_row_ptr[e * N:(e + 1) * N + 1]
        single = oracle.gemv(mode, bits, N, K, W.indices[e], W.codebooks[e],
                             None if W.group_ids is None else W.group_ids[e],
                             rp - rp[0], W.out_col[rp[0]:rp[-1]], W.out_val[rp[0]:rp[-1]], xt[t])
        assert np.array_equal(y_slot[t], single[0])
    assert oracle.gemv_moe(W, np.zeros(0, np.int32), xs, shared_x=True).shape == (0, N)
    with pytest.raises(ValueError):
        oracle.gemv_moe(W, np.array([E], np.int32), xs, shared_x=True)


def test_a_dropped_term_would_exceed_the_gate():
    # the 1e-3 gate is meaningful: losing one bulk term or one outlier is visible
    W = xi.config_weights(1)
    x = xi.config_x(1, 1, W.K)
    y = oracle.gemv_weights(W, x)
    C, O = np_dense_weight(W)
    xd = x.view(np.float16).astype(np.float64)
    worst_bulk = np.abs(C[0] * xd[0]).max()
    y_bad = y.copy()
    y_bad[0, 0] -= worst_bulk
    assert gated_rel_err(y_bad, y) > 1e-3
    j = W.out_row_ptr[np.argmax(np.diff(W.out_row_ptr) > 0)]
    n = np.searchsorted(W.out_row_ptr, j, side="right") - 1
    y_bad = y.copy()
    y_bad[0, n] -= float(W.out_val[j:j + 1].view(np.float16)[0]) * xd[0, W.out_col[j]]
    assert gated_rel_err(y_bad, y) > 1e-3


def test_silu_mul_against_library_logistic_closed_forms_and_layout():
    # SiLU(g) = g * logistic(g): scipy's expit is an independent routine for the logistic function
    from scipy.special import expit
    rng = np.random.default_rng(5)
    y = rng.normal(0.0, 3.0, size=(4, 10))
    h = oracle.silu_mul(y)
    assert h.shape == (4, 5)
    assert np.allclose(h, y[:, :5] * expit(y[:, :5]) * y[:, 5:], rtol=1e-14, atol=0.0)
    # closed forms: SiLU(0) = 0; SiLU(g) - SiLU(-g) = g; SiLU(g) -> g for large g, -> 0 for very negative g
    z = oracle.silu_mul(np.array([0.0, 7.0, -7.0, 50.0, -800.0, 1.0, 1.0, 1.0, 1.0, 1.0]))
    assert z[0] == 0.0 and abs((z[1] - z[2]) - 7.0) < 1e-14
    assert abs(z[3] - 50.0) < 1e-12 and z[4] == 0.0
    # SiLU(1) = 1 / (1 + 1/e)
    assert abs(oracle.silu_mul(np.array([1.0, 2.0]))[0] - 2.0 / (1.0 + np.exp(-1.0))) < 1e-15
    # layout: gate rows first, up rows second; swapping them changes the result (silu is not symmetric)
    w = np.array([[2.0, -1.0, 0.5, 3.0]])
    assert np.allclose(oracle.silu_mul(w), [[2.0 * expit(2.0) * 0.5, -expit(-1.0) * 3.0]])
    assert not np.allclose(oracle.silu_mul(w), oracle.silu_mul(w[:, [2, 3, 0, 1]]))


def test_moe_combine_special_cases_and_matmul():
    rng = np.random.default_rng(9)
    y = rng.normal(size=(5, 12))
    w = rng.random(5).astype(np.float32)
    assert np.allclose(oracle.moe_combine(y, w), w.astype(np.float64) @ y, rtol=1e-14)        # library matmul
    e = np.zeros(5, np.float32)
    e[3] = 1.0
    assert np.array_equal(oracle.moe_combine(y, e), y[3])                                      # one-hot picks a slot
    assert np.array_equal(oracle.moe_combine(y, np.zeros(5, np.float32)), np.zeros(12))
    assert np.allclose(oracle.moe_combine(y, np.full(5, 0.5, np.float32)), 0.5 * y.sum(axis=0), rtol=1e-14)
    # linear in the weights and in y
    w2 = rng.random(5).astype(np.float32)
    assert np.allclose(oracle.moe_combine(y, w) + oracle.moe_combine(y, w2),
                       (w.astype(np.float64) + w2.astype(np.float64)) @ y, rtol=1e-13)
    assert np.allclose(oracle.moe_combine(y + 2.0 * y[::-1], w), oracle.moe_combine(y, w) + 2.0 * oracle.moe_combine(y[::-1], w),
                       rtol=1e-13)


# ------------------------------------------------------------------ 5 and 6 bits; the word forms of the packing table
def test_unpack_hand_vectors_5_and_6_bit_dense_stream():
    # 5-bit: field 6 = 21 = 0b10101 occupies stream bits 30..34: bits 30, 31 of word 0 (1, 0) and bits 0..2 of
    # word 1 (1, 0, 1); field 0 = 31
    words = np.array([[0x4000001F, 0x00000005, 0, 0, 0]], dtype=np.uint32)
    exp = np.zeros((1, 32), dtype=np.uint8)
    exp[0, 0], exp[0, 6] = 31, 21
    assert np.array_equal(oracle.unpack(words, 32, 5), exp)
    assert np.array_equal(oracle.pack(exp, 5), words)
    # 6-bit: field 5 = 0b110011 = 51 occupies stream bits 30..35: word 0 bits 30, 31 = (1, 1), word 1 bits 0..3 = (0, 0, 1, 1)
    words = np.array([[0xC0000000, 0x0000000C, 0]], dtype=np.uint32)
    exp = np.zeros((1, 16), dtype=np.uint8)
    exp[0, 5] = 51
    assert np.array_equal(oracle.unpack(words, 16, 6), exp)


@pytest.mark.parametrize("bits", [5, 6])
def test_pack_unpack_round_trip_5_and_6_bit(bits):
    rng = np.random.default_rng(bits)
    q = rng.integers(0, 1 << bits, size=(7, 384), dtype=np.uint8)
    w = oracle.pack(q, bits)
    assert w.shape == (7, 384 * bits // 32)
    assert np.array_equal(oracle.unpack(w, 384, bits), q)
    assert np.array_equal(np_unpack(w, 384, bits), q)                          # numpy bit expansion
    assert all(np.array_equal(bigint_pack(q[r], bits), w[r]) for r in range(7))   # big-integer packer


def test_word_forms_hand_written():
    # 5 bits: three values per uint16, bit 15 reserved.  (31, 0, 21) -> 31 | 21 << 10 = 0x541F; with the reserve bit
    # set the same three values must come out
    for word in (0x541F, 0xD41F):
        assert oracle.unpack_wordform(np.array([[word]], np.uint16), 3, 5).tolist() == [[31, 0, 21]]
    # 6 bits: five per uint32, bits 30, 31 reserved.  (1, 2, 3, 4, 63) -> 1 | 2<<6 | 3<<12 | 4<<18 | 63<<24
    w6 = 1 | 2 << 6 | 3 << 12 | 4 << 18 | 63 << 24
    assert w6 == 0x3F103081
    for word in (w6, w6 | 0xC0000000):
        assert oracle.unpack_wordform(np.array([[word]], np.uint32), 5, 6).tolist() == [[1, 2, 3, 4, 63]]
    # 3 bits through the general routine = the ten-per-word routine
    w3 = np.array([[0o1234567012 | 0x80000000, 0o7]], np.uint32)
    assert np.array_equal(oracle.unpack_wordform(w3, 11, 3), oracle.unpack_word10(w3, 11))
    # a part-filled last word: K = 4 at 5 bits takes two uint16
    assert oracle.unpack_wordform(np.array([[0x541F, 0x0007]], np.uint16), 4, 5).tolist() == [[31, 0, 21, 7]]


def test_word_forms_match_the_packing_table_counts():
    per_word = {}
    for line in open(GOLDEN):
        t = line.split("#")[0].split()
        if t and t[0] == "pack":
            n, per, wbits, used, reserve = map(int, t[1:])
            assert per * n == used and used + reserve == wbits
            per_word[n] = (per, wbits)
    rng = np.random.default_rng(11)
    for bits, (per, wbits) in per_word.items():
        K = 256
        q = rng.integers(0, 1 << bits, size=(3, K), dtype=np.uint8)
        w = xi.pack_wordform(q, bits)                                          # the generator's own packer
        assert w.dtype.itemsize * 8 == wbits and w.shape == (3, -(-K // per))
        assert np.array_equal(oracle.unpack_wordform(w, K, bits), q)
        assert np.array_equal(oracle.repack_wordform(w, K, bits), oracle.pack(q, bits))
        if bits in (2, 4):                                                     # no reserve bits: the word form IS the dense stream
            assert np.array_equal(w, oracle.pack(q, bits))


# ------------------------------------------------------------------ V2a with a scale and a mid-point per group
def test_affine_groups_identity_is_the_plain_library():
    W = xi.random_weights(V2A, 4, 12, 512, density=0.004, seed=40, affine=True)
    x = xi.activations(np.random.default_rng(41), 3, W.K)
    plain = oracle.gemv(V2A, 4, W.N, W.K, W.indices[0], W.codebooks[0], W.group_ids[0], W.out_row_ptr, W.out_col, W.out_val, x)
    one, zero = np.full_like(W.group_scale[0], 0x3C00), np.zeros_like(W.group_mid[0])
    ident = oracle.gemv(V2A, 4, W.N, W.K, W.indices[0], W.codebooks[0], W.group_ids[0], W.out_row_ptr, W.out_col, W.out_val, x,
                        group_scale=one, group_mid=zero)
    assert np.array_equal(plain, ident)
    assert not np.allclose(plain, oracle.gemv_weights(W, x))                   # the generated scales and mid-points do act


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_affine_groups_against_dense_numpy_and_exact_rationals(bits):
    from fractions import Fraction
    W = xi.random_weights(V2A, bits, 9, 384, L=7, density=0.01, seed=50 + bits, affine=True)
    x = xi.activations(np.random.default_rng(51), 2, W.K)
    # dense build with numpy fancy indexing (not the oracle's loop): C * scale + mid per group, plus the outliers
    C, O = np_dense_weight(W)
    s = np.repeat(W.group_scale[0].view(np.float16).astype(np.float64), 128, axis=1)
    m = np.repeat(W.group_mid[0].view(np.float16).astype(np.float64), 128, axis=1)
    dense = C * s + m + O
    xf = x.view(np.float16).astype(np.float64)
    got = oracle.gemv_weights(W, x)
    assert gated_rel_err(got, xf @ dense.T) <= 1e-12
    # the dequantised doubles themselves, and one output in exact rational arithmetic
    _, wd = oracle.dequant_bulk(V2A, bits, W.N, W.K, W.indices[0], W.codebooks[0], W.group_ids[0],
                                group_scale=W.group_scale[0], group_mid=W.group_mid[0])
    assert np.array_equal(wd, C * s + m)
    n = 4
    exact = sum(Fraction(float(xf[1, k])) * (Fraction(float(C[n, k])) * Fraction(float(s[n, k])) + Fraction(float(m[n, k])) + Fraction(float(O[n, k])))
                for k in range(W.K))
    assert abs(got[1, n] - float(exact)) <= 1e-12 * max(1.0, abs(float(exact)))
    # the mid-point alone: zero codebooks, unit scale -> y[n] = sum_g mid[n, g] * (sum of x over group g)
    Z = xi.random_weights(V2A, bits, 9, 384, L=7, density=0.0, seed=60, affine=True)
    Z.codebooks[:] = 0
    yz = oracle.gemv_weights(Z, x)
    xs = xf.reshape(2, 3, 128).sum(axis=2)
    assert gated_rel_err(yz, xs @ Z.group_mid[0].view(np.float16).astype(np.float64).T) <= 1e-12


def test_affine_groups_expert_indexed_slices_scale_and_mid_by_expert():
    W = xi.random_weights(V2A, 3, 6, 256, E=3, density=0.01, seed=70, affine=True)
    x = xi.activations(np.random.default_rng(71), 1, W.K)
    ids = np.array([2, 0, 2], np.int32)
    y = oracle.gemv_moe(W, ids, x, shared_x=True)
    for t, e in enumerate(ids):
        rp = W.out_row_ptr[e * W.N:(e + 1) * W.N + 1]
        single = oracle.gemv(V2A, 3, W.N, W.K, W.indices[e], W.codebooks[e], W.group_ids[e], rp, W.out_col, W.out_val, x,
                             group_scale=W.group_scale[e], group_mid=W.group_mid[e])
        assert np.array_equal(y[t], single[0])
