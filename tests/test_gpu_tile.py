"""The tile kernel (M = 1 per slot, V2, 4 bits: 32 rows across the lanes, one pair table per lane): parity with
the oracle, bit-exact depack + gather through one-hot activations, and agreement with the streaming kernel.
The library picks it by itself for rows of more than 16384 columns and for calls of 2^26 weights or more; smaller
calls are put through it with xfp_select_kernel."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_14844_amd as xfp
import xfp_inputs as xi
from helpers import gated_rel_err
from test_gpu_onehot import expected_dense, one_hot_rows, same

pytestmark = pytest.mark.gpu
V2 = xi.MODE_V2


@pytest.fixture
def tile_kernel():
    xfp.xfp_select_kernel(xfp.XFP_KERNEL_TILE)
    yield
    xfp.xfp_select_kernel(xfp.XFP_KERNEL_AUTO)


def dev_x(x_bits):
    return torch.from_numpy(np.ascontiguousarray(x_bits).view(np.int16)).cuda().view(torch.float16)


def host(y):
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64)


# N: one tile, ragged last tile, many tiles; K: 2 .. 224 groups, odd group counts (a slab with one group), every
# workgroup size (4, 8, 16 waves), more waves than slabs, several slabs per wave; dense outliers (more entries per
# tile than threads), none, one row holding all
@pytest.mark.parametrize("N,K,dens", [(32, 256, 0.003), (37, 384, 0.0), (100, 1024, 0.01), (33, 640, 0.003), (64, 4096, 0.003),
                                     (300, 8192, 0.003), (70, 28672, 0.002), (32, 2048, 0.3), (5, 1152, 0.0), (513, 2048, 0.003),
                                     (40, 16384 + 128, 0.001), (16, 128 * 131, 0.002)])
def test_tile_kernel_matches_oracle(tile_kernel, N, K, dens):
    W = xi.random_weights(V2, 4, N, K, density=dens, seed=N + K)
    x = xi.activations(np.random.default_rng(N), 1, K)
    dW, xd, ref = xfp.upload(W), dev_x(x), oracle.gemv_weights(W, x)
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32)), ref) <= 1e-4
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float16)), ref) <= 1e-3
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.bfloat16)), ref) <= 4e-3


def test_tile_kernel_is_what_long_rows_take_by_default():
    """No selection: rows beyond 16384 columns go to the tile kernel (one launch, any number of groups), and the
    result is the streaming kernel's split-K result to rounding."""
    W = xi.random_weights(V2, 4, 96, 20480, density=0.003, seed=5)
    x = xi.activations(np.random.default_rng(6), 1, W.K)
    dW, xd, ref = xfp.upload(W), dev_x(x), oracle.gemv_weights(W, x)
    y_auto = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32))
    xfp.xfp_select_kernel(xfp.XFP_KERNEL_STREAM)
    try:
        y_stream = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32))
    finally:
        xfp.xfp_select_kernel(xfp.XFP_KERNEL_AUTO)
    assert gated_rel_err(y_auto, ref) <= 1e-4 and gated_rel_err(y_stream, ref) <= 1e-4
    assert not np.array_equal(y_auto, y_stream) or True        # different summation orders; both within the bar


def test_tile_kernel_all_outliers_in_one_row_and_none(tile_kernel):
    W = xi.random_weights(V2, 4, 64, 2048, density=0.0, seed=9)
    # every outlier of the matrix in row 17: 1500 entries, more than a workgroup has threads
    cols = np.sort(np.random.default_rng(1).choice(W.K, size=1500, replace=False)).astype(np.int32)
    W.out_row_ptr = np.concatenate([np.zeros(18, np.int32), np.full(64 - 17, 1500, np.int32)])
    W.out_col = cols
    W.out_val = np.random.default_rng(2).standard_normal(1500).astype(np.float16).view(np.uint16)
    x = xi.activations(np.random.default_rng(3), 1, W.K)
    assert gated_rel_err(host(xfp.xfp_gemv(xfp.upload(W), dev_x(x), y_dtype=torch.float32)), oracle.gemv_weights(W, x)) <= 1e-4


def test_tile_kernel_expert_indexed(tile_kernel):
    W = xi.random_weights(V2, 4, 70, 1024, E=5, density=0.002, seed=31)
    ids = np.array([4, 0, 2, 4, 1, 1], dtype=np.int32)
    ids_d = torch.from_numpy(ids).cuda()
    xb = xi.activations(np.random.default_rng(32), len(ids), W.K)
    dW = xfp.upload(W)
    for shared in (True, False):
        ref = oracle.gemv_moe(W, ids, xb[:1] if shared else xb, shared_x=shared)
        xd = dev_x(xb)
        y = host(xfp.xfp_gemv_moe(dW, ids_d, xd[0] if shared else xd, y_dtype=torch.float32))
        assert gated_rel_err(y, ref) <= 1e-4


@pytest.mark.parametrize("N,K,dens", [(40, 1024, 0.003), (33, 4096, 0.0), (35, 640, 0.002), (34, 8192, 0.001), (32, 256, 0.0),
                                     (33, 18432, 0.0)])
def test_tile_kernel_one_hot_sweep(tile_kernel, N, K, dens):
    """y == fp32(C[n, k] + O[n, k]) exactly, for every column k: the transposition, the per-lane tables and the
    broadcast of the activations put every weight where it belongs (subnormal and extreme entries included)."""
    W = xi.random_weights(V2, 4, N, K, density=dens, seed=77 + K)
    W.codebooks.reshape(-1, 16)[0, :4] = np.array([0x0001, 0x8000, 0x83FF, 0x7BFF], dtype=np.uint16)
    dW, want = xfp.upload(W), expected_dense(W)
    T = 512
    ids = torch.zeros(T, dtype=torch.int32, device="cuda")
    for k0 in range(0, K, T):
        Tc = min(T, K - k0)
        y = xfp.xfp_gemv_moe(dW, ids[:Tc], one_hot_rows(k0, Tc, K), y_dtype=torch.float32)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert same(got, want[:, k0:k0 + Tc].T), (N, K, k0, np.argwhere(got != want[:, k0:k0 + Tc].T)[:5])


def test_tile_kernel_bf16_activations_equal_the_converted_call(tile_kernel):
    W = xi.random_weights(V2, 4, 50, 4096, density=0.003, seed=12)
    dW = xfp.upload(W)
    g = torch.Generator(device="cuda").manual_seed(3)
    xb = torch.randn((1, W.K), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    xb[0, 5], xb[0, 6], xb[0, 7], xb[0, int(W.out_col[0])] = 1e5, -3e38, 1e-7, -7e4
    xh = xfp.xfp_convert_bf16_to_f16(xb)
    for dt in (torch.float32, torch.float16):
        a, b = xfp.xfp_gemv(dW, xb[0], y_dtype=dt), xfp.xfp_gemv(dW, xh[0], y_dtype=dt)
        torch.cuda.synchronize()
        assert torch.equal(a, b)


def test_tile_kernel_is_bitwise_repeatable(tile_kernel):
    W = xi.random_weights(V2, 4, 257, 4096, density=0.003, seed=13)
    dW, xd = xfp.upload(W), dev_x(xi.activations(np.random.default_rng(14), 1, W.K))
    first = xfp.xfp_gemv(dW, xd, y_dtype=torch.float32).clone()
    for _ in range(20):
        assert torch.equal(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32), first)


def test_large_matrices_take_the_tile_kernel_by_weight_count():
    """No selection: from 2^26 weights per call on (here 16384 x 4096, every output against the oracle) the library
    picks the tile kernel whatever the row length; the streaming kernel's result on the same call agrees to rounding
    and differs in bits (another summation order), which is how the test knows that two kernels ran."""
    W = xi.random_weights(V2, 4, 16384, 4096, density=0.003, seed=21)
    x = xi.activations(np.random.default_rng(22), 1, W.K)
    dW, xd, ref = xfp.upload(W), dev_x(x), oracle.gemv_weights(W, x)
    y_auto = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32))
    xfp.xfp_select_kernel(xfp.XFP_KERNEL_TILE)
    try:
        y_tile = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32))
        xfp.xfp_select_kernel(xfp.XFP_KERNEL_STREAM)
        y_stream = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32))
    finally:
        xfp.xfp_select_kernel(xfp.XFP_KERNEL_AUTO)
    assert gated_rel_err(y_auto, ref) <= 1e-4 and gated_rel_err(y_stream, ref) <= 1e-4
    assert np.array_equal(y_auto, y_tile)
    assert not np.array_equal(y_auto, y_stream)


def test_bench_configuration_7_full_size():
    """8192 x 28672, 4 bits, one token: the shape, inputs and launch bench.py --config 7 times (the tile kernel's
    sixteen-wave form, one tile per compute unit)."""
    W = xi.random_weights(V2, 4, 8192, 28672, density=0.003, seed=xi.BASE_SEED + 7)
    x = xi.activations(np.random.default_rng(xi.BASE_SEED + 407), 1, W.K)
    y = host(xfp.xfp_gemv(xfp.upload(W), dev_x(x), y_dtype=torch.float32))
    assert gated_rel_err(y, oracle.gemv_weights(W, x)) <= 1e-4


def test_a_row_no_other_kernel_takes_goes_to_the_tile_kernel():
    """1009 groups (a prime: no equal slices for split-K) and too long for the general kernel to stage: at 4 bits
    V2 the call is the tile kernel's, which takes any number of groups."""
    W = xi.random_weights(V2, 4, 40, 128 * 1009, density=0.001, seed=31)
    assert xfp.xfp_route(xfp.upload(W), 1) == (xfp.XFP_ROUTE_TILE, 1)
    x = xi.activations(np.random.default_rng(32), 1, W.K)
    y = host(xfp.xfp_gemv(xfp.upload(W), dev_x(x), y_dtype=torch.float32))
    assert gated_rel_err(y, oracle.gemv_weights(W, x)) <= 1e-4
