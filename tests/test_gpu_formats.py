"""The formats beyond the five workloads (paper sections 3.1, 3.3 and 3.4): 5- and 6-bit indices, the word
forms of the packing table converted at load, and V2a matrices with a scale and a mid-point per group.  All of
them run the general kernel; bars as everywhere: bit-exact for indices and dequantised patterns, 1e-4 gated for
fp32 outputs, 1e-3 for fp16."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_14844_amd as xfp
import xfp_inputs as xi
from helpers import gated_rel_err
from test_gpu_onehot import one_hot_rows, same

pytestmark = pytest.mark.gpu
V2, V2A = xi.MODE_V2, xi.MODE_V2A


def dev_x(x_bits):
    return torch.from_numpy(np.ascontiguousarray(x_bits).view(np.int16)).cuda().view(torch.float16)


def host(y):
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("mode,bits,N,K,E", [(V2, 5, 37, 384, 1), (V2, 6, 70, 1024, 1), (V2A, 5, 33, 2048, 1), (V2A, 6, 19, 128, 2),
                                             (V2, 5, 16, 256, 3)])
def test_unpack_and_dequant_bit_exact_5_and_6_bits(mode, bits, N, K, E):
    W = xi.random_weights(mode, bits, N, K, E=E, density=0.002, seed=bits * 1000 + N)
    dW = xfp.upload(W)
    q = xfp.xfp_unpack_indices(dW).cpu().numpy()
    assert np.array_equal(q, oracle.unpack(W.indices, K, bits).reshape(E * N, K))
    w = xfp.xfp_dequant_bulk(dW).cpu().numpy().view(np.uint16)
    for e in range(E):
        ref, _ = oracle.dequant_bulk(mode, bits, N, K, W.indices[e], W.codebooks[e],
                                     None if W.group_ids is None else W.group_ids[e], want_double=False)
        assert np.array_equal(w[e * N:(e + 1) * N], ref)


@pytest.mark.parametrize("bits", [2, 3, 4, 5, 6])
@pytest.mark.parametrize("rows,K", [(1, 128), (37, 384), (70, 4096)])
def test_repack_words_bit_exact(bits, rows, K):
    rng = np.random.default_rng(rows + K + bits)
    q = rng.integers(0, 1 << bits, size=(rows, K), dtype=np.uint8)
    w = xi.pack_wordform(q, bits)
    reserve = {2: 0, 3: 2, 4: 0, 5: 1, 6: 2}[bits]
    if reserve:                                                # whatever sits in the reserve bits must not matter
        top = w.dtype.itemsize * 8 - reserve
        w = w | (rng.integers(0, 1 << reserve, size=w.shape).astype(w.dtype) << w.dtype.type(top))
    t = torch.from_numpy(w.view(np.int16 if bits == 5 else np.int32)).cuda()
    got = xfp.xfp_repack_words(t, K, bits)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint32), oracle.repack_wordform(w, K, bits))
    assert np.array_equal(got.cpu().numpy().view(np.uint32), oracle.pack(q, bits))


@pytest.mark.parametrize("mode,bits,N,K,M", [(V2, 5, 100, 1024, 1), (V2, 6, 65, 4096, 1), (V2A, 5, 40, 2048, 1), (V2A, 6, 33, 640, 1),
                                             (V2, 5, 50, 8192, 5), (V2, 6, 24, 20480, 1), (V2, 5, 30, 384, 17)])
def test_gemv_5_and_6_bits_matches_oracle(mode, bits, N, K, M):
    W = xi.random_weights(mode, bits, N, K, density=0.003, seed=N + K + bits)
    x = xi.activations(np.random.default_rng(N), M, K)
    dW, xd, ref = xfp.upload(W), dev_x(x), oracle.gemv_weights(W, x)
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32)), ref) <= 1e-4
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float16)), ref) <= 1e-3


def test_expert_indexed_calls_and_epilogues_at_6_bits():
    W = xi.random_weights(V2, 6, 48, 1024, E=4, density=0.002, seed=3)
    rng = np.random.default_rng(4)
    ids = np.array([3, 0, 0, 2, 1], np.int32)
    ids_d = torch.from_numpy(ids).cuda()
    xb = xi.activations(rng, len(ids), W.K)
    dW, xd = xfp.upload(W), dev_x(xb)
    ref = oracle.gemv_moe(W, ids, xb, shared_x=False)
    assert gated_rel_err(host(xfp.xfp_gemv_moe(dW, ids_d, xd, y_dtype=torch.float32)), ref) <= 1e-4
    assert gated_rel_err(host(xfp.xfp_gemv_moe_silu_mul(dW, ids_d, xd, h_dtype=torch.float32)), oracle.silu_mul(ref)) <= 1e-4
    w = rng.random(len(ids)).astype(np.float32)
    y = host(xfp.xfp_gemv_moe_combine(dW, ids_d, xd, torch.from_numpy(w).cuda(), y_dtype=torch.float32))
    assert gated_rel_err(y[None, :], oracle.moe_combine(ref, w)[None, :]) <= 1e-4


@pytest.mark.parametrize("bits,N,K", [(5, 6, 512), (6, 5, 1152)])
def test_general_kernel_one_hot_sweep_5_and_6_bits(bits, N, K):
    """y == fp32(C[n, k] + O[n, k]) exactly for every column: every word-straddling 5- and 6-bit field."""
    from test_gpu_onehot import expected_dense
    W = xi.random_weights(V2, bits, N, K, density=0.002, seed=bits)
    dW, want = xfp.upload(W), expected_dense(W)
    ids = torch.zeros(K, dtype=torch.int32, device="cuda")
    y = xfp.xfp_gemv_moe(dW, ids, one_hot_rows(0, K, K), y_dtype=torch.float32)
    torch.cuda.synchronize()
    assert same(y.cpu().numpy(), want.T)


# ------------------------------------------------------------------ V2a with a scale and a mid-point per group
@pytest.mark.parametrize("bits,N,K,M,E", [(4, 100, 1024, 1, 1), (3, 65, 4096, 1, 1), (2, 40, 2048, 3, 1), (4, 33, 640, 18, 1),
                                          (4, 24, 20480, 1, 1), (5, 20, 512, 1, 1)])
def test_affine_groups_match_oracle(bits, N, K, M, E):
    W = xi.random_weights(V2A, bits, N, K, density=0.003, seed=N + K + bits, affine=True)
    x = xi.activations(np.random.default_rng(N), M, K)
    dW, xd, ref = xfp.upload(W), dev_x(x), oracle.gemv_weights(W, x)
    assert dW.desc.flags == 1
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32)), ref) <= 1e-4
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float16)), ref) <= 1e-3
    # and the affine map does act: the same call without the two arrays differs
    W.group_scale = W.group_mid = None
    assert gated_rel_err(host(xfp.xfp_gemv(xfp.upload(W), xd, y_dtype=torch.float32)), ref) > 1e-2


def test_affine_groups_identity_equals_the_plain_library():
    """Scale 1 and mid-point 0: s * u + 0 * xs is u exactly; what remains is the order of the fp32 sums (per unit
    first in the affine form), far inside the fp32 bar."""
    W = xi.random_weights(V2A, 4, 64, 20480 + 128 * 3, density=0.002, seed=8, affine=True)   # 163 groups (prime): the general kernel either way
    x = xi.activations(np.random.default_rng(9), 1, W.K)
    xd = dev_x(x)
    W.group_scale[:] = 0x3C00
    W.group_mid[:] = 0
    a = xfp.xfp_gemv(xfp.upload(W), xd, y_dtype=torch.float32)
    W.group_scale = W.group_mid = None
    b = xfp.xfp_gemv(xfp.upload(W), xd, y_dtype=torch.float32)
    torch.cuda.synchronize()
    assert gated_rel_err(host(a), host(b)) <= 1e-4


def test_affine_groups_one_hot_is_the_exact_affine_value():
    """One-hot x, no outliers: y[n] == fp32(entry * scale + mid) with ONE rounding (a fused multiply-add of exact
    operands), against the oracle's doubles rounded once."""
    W = xi.random_weights(V2A, 4, 6, 512, L=9, density=0.0, seed=10, affine=True)
    _, wd = oracle.dequant_bulk(V2A, 4, W.N, W.K, W.indices[0], W.codebooks[0], W.group_ids[0],
                                group_scale=W.group_scale[0], group_mid=W.group_mid[0])
    dW = xfp.upload(W)
    ids = torch.zeros(W.K, dtype=torch.int32, device="cuda")
    y = xfp.xfp_gemv_moe(dW, ids, one_hot_rows(0, W.K, W.K), y_dtype=torch.float32)
    torch.cuda.synchronize()
    assert same(y.cpu().numpy(), wd.astype(np.float32).T)


def test_affine_groups_expert_indexed():
    W = xi.random_weights(V2A, 3, 40, 1024, E=3, density=0.002, seed=11, affine=True)
    ids = np.array([2, 0, 2, 1], np.int32)
    xb = xi.activations(np.random.default_rng(12), len(ids), W.K)
    ref = oracle.gemv_moe(W, ids, xb, shared_x=False)
    y = host(xfp.xfp_gemv_moe(xfp.upload(W), torch.from_numpy(ids).cuda(), dev_x(xb), y_dtype=torch.float32))
    assert gated_rel_err(y, ref) <= 1e-4


# ------------------------------------------------------------------ matrices written by the reference encoder
@pytest.mark.parametrize("mode,bits,N,K", [(V2, 4, 300, 4096), (V2, 3, 130, 1024), (V2, 2, 64, 2048), (V2, 4, 40, 20480),
                                           (V2A, 4, 96, 1024), (V2A, 2, 70, 512)])
def test_decode_of_what_the_reference_encoder_writes(mode, bits, N, K):
    """Heavy-tailed weights through outlier extraction, Lloyd codebooks (V2) or LibFit with a scale and a mid-point
    per group (V2a): non-uniform index histograms, residual outliers.  The decoded product must match the oracle
    AND the exact product with the original weights to the encoder's own cosine."""
    import xfp_encoder as enc
    Wf = 0.02 * np.random.default_rng(N + K).standard_t(4.0, size=(N, K))
    e = (enc.encode_v2 if mode == V2 else enc.encode_v2a)(Wf, bits)
    x = xi.activations(np.random.default_rng(K), 1, K)
    dW, xd, ref = xfp.upload(e.weights), dev_x(x), oracle.gemv_weights(e.weights, x)
    y = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32))
    assert gated_rel_err(y, ref) <= 1e-4
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float16)), ref) <= 1e-3
    exact = x.view(np.float16).astype(np.float64) @ Wf.T
    cos = float((y * exact).sum() / np.sqrt((y * y).sum() * (exact * exact).sum()))
    assert cos > {2: 0.9, 3: 0.97, 4: 0.99}[bits]


@pytest.mark.parametrize("bits,N,K,M,L", [(3, 4096, 4096, 1, 32), (4, 100, 2048, 3, 32), (2, 65, 16384, 1, 7), (4, 33, 5120, 2, 63),
                                          (3, 20, 640, 5, 200), (4, 40, 1024, 1, 1), (2, 257, 12288, 1, 256)])
def test_affine_groups_through_the_streaming_kernel(bits, N, K, M, L):
    """Rows the streaming kernel holds (up to 16384 columns, short rows in its tail form): the call takes that
    kernel's mode for flagged tensors, token by token, and matches the oracle; C3's shape among them."""
    W = xi.random_weights(V2A, bits, N, K, L=L, density=0.002, seed=N + K + bits + L, affine=True)
    dW = xfp.upload(W)
    assert xfp.xfp_route(dW, M) == (xfp.XFP_ROUTE_STREAM, M)
    x = xi.activations(np.random.default_rng(N + M), M, K)
    xd, ref = dev_x(x), oracle.gemv_weights(W, x)
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32)), ref) <= 1e-4
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float16)), ref) <= 1e-3
    xb = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16).float().bfloat16()          # bf16 activations: the
    want = xfp.xfp_gemv(dW, xfp.xfp_convert_bf16_to_f16(xb), y_dtype=torch.float32)                 # converted call's bits
    assert torch.equal(xfp.xfp_gemv(dW, xb, y_dtype=torch.float32), want)
