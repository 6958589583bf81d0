"""The wide matrix-core kernel (V2 and V2a, 2 to 4 bits, 17 .. 64 tokens in one pass over the weights): parity with the oracle,
bit-exact depack + gather through one-hot activations, agreement with the single-token calls, the token counts and
row lengths at which the call falls back to chunks of 16."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_14844_amd as xfp
import xfp_inputs as xi
from helpers import gated_rel_err

pytestmark = pytest.mark.gpu
V2, V2A = xi.MODE_V2, xi.MODE_V2A


def dev_x(x_bits):
    return torch.from_numpy(np.ascontiguousarray(x_bits).view(np.int16)).cuda().view(torch.float16)


def host(y):
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64)


def check(W, x, tol32=1e-4, tol16=1e-3):
    dW, xd, ref = xfp.upload(W), dev_x(x), oracle.gemv_weights(W, x)
    y32 = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32))
    y16 = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float16))
    e32, e16 = gated_rel_err(y32, ref), gated_rel_err(y16, ref)
    print(f"  N={W.N} K={W.K} M={x.shape[0]}: err f32 {e32:.2e} f16 {e16:.2e}", flush=True)
    assert e32 <= tol32 and e16 <= tol16
    return dW, xd, ref, y32


# N: one tile, a ragged last tile, rows that leave the second row block empty, many tiles; K: fewer groups than
# waves, a group count that is no multiple of 8, the longest row 64 tokens go with (8192), longer rows with fewer
# tokens; M: every chunk count, full and ragged last chunks; outliers: none, the benchmark's density, dense
@pytest.mark.parametrize("N,K,M,dens", [(32, 1024, 64, 0.003), (77, 4096, 17, 0.003), (200, 8192, 64, 0.003),
                                        (10, 384, 33, 0.01), (45, 2176, 48, 0.0), (129, 5120, 32, 0.003),
                                        (64, 16384, 32, 0.003), (40, 10880, 47, 0.003), (33, 128, 20, 0.05),
                                        (300, 7296, 49, 0.02), (4500, 256, 64, 0.003)])
@pytest.mark.parametrize("bits", [4, 3, 2])
@pytest.mark.parametrize("mode", [V2, V2A])
def test_wide_kernel_matches_oracle(mode, bits, N, K, M, dens):
    W = xi.random_weights(mode, bits, N, K, density=dens, seed=N + K + M)
    check(W, xi.activations(np.random.default_rng(M + N), M, K))


@pytest.mark.parametrize("bits,L", [(4, 64), (4, 65), (4, 1), (3, 256), (3, 5), (2, 256), (2, 2)])
def test_wide_kernel_library_sizes(bits, L):
    """Libraries up to the 64 KB of pair tables the kernel holds; 65 codebooks at 4 bits are one too many and go
    token by token."""
    W = xi.random_weights(V2A, bits, 70, 2048, L=L, density=0.003, seed=L + bits)
    fits = (L << (2 * bits)) * 4 <= 65536
    assert (xfp.xfp_route(xfp.upload(W), 40)[0] == xfp.XFP_ROUTE_WIDE) == fits
    check(W, xi.activations(np.random.default_rng(L), 40, 2048))


def test_wide_kernel_agrees_with_single_token_calls_and_is_repeatable():
    W = xi.random_weights(V2, 4, 150, 4096, density=0.003, seed=3)
    x = xi.activations(np.random.default_rng(4), 40, W.K)
    dW, xd, ref, y = check(W, x)
    for m in (0, 15, 16, 39):
        y1 = host(xfp.xfp_gemv(dW, xd[m:m + 1].contiguous(), y_dtype=torch.float32))
        assert gated_rel_err(y[m], y1[0]) <= 1e-4
    first = xfp.xfp_gemv(dW, xd, y_dtype=torch.float32).clone()
    for _ in range(10):
        assert torch.equal(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32), first)


def test_wide_kernel_one_row_holds_every_outlier():
    """All entries in one row (more than two 64-entry chunks of a wave's run), none elsewhere."""
    W = xi.random_weights(V2, 4, 70, 2048, density=0.0, seed=9)
    cols = np.sort(np.random.default_rng(1).choice(W.K, size=700, replace=False)).astype(np.int32)
    W.out_row_ptr = np.concatenate([np.zeros(38, np.int32), np.full(70 - 37, 700, np.int32)])
    W.out_col = cols
    W.out_val = xi.activations(np.random.default_rng(2), 1, 700).ravel()
    check(W, xi.activations(np.random.default_rng(3), 24, W.K))


@pytest.mark.parametrize("mode,bits,N,K,M", [(V2, 4, 48, 1024, 64), (V2, 4, 37, 640, 19), (V2, 3, 48, 1024, 64), (V2, 3, 37, 640, 35),
                                             (V2, 2, 40, 768, 64), (V2A, 4, 45, 1152, 64), (V2A, 3, 37, 640, 35),
                                             (V2A, 2, 50, 768, 48)])
def test_wide_kernel_one_hot_sweep(mode, bits, N, K, M):
    """Token m carries a single 1.0 at column (k0 + m) of a sweep over all columns: y[m][n] must then be EXACTLY the
    dequantized weight Codebook[n][q[n, k]] (+ the outlier at that position), bit for bit: the kernel's own depack
    and gather, not the stand-alone hooks', are what is checked."""
    W = xi.random_weights(mode, bits, N, K, density=0.01, seed=N + K)
    dW = xfp.upload(W)
    q = oracle.unpack(W.indices[0], K, bits).astype(np.int64)
    cb = W.codebooks[0].view(np.float16).astype(np.float32)                     # V2 [N][2^bits], V2a [L][2^bits]
    if mode == V2:
        dense = np.take_along_axis(cb, q, axis=1)                               # [N][K]
    else:
        dense = cb[np.repeat(W.group_ids[0].astype(np.int64), 128, axis=1), q]  # the group's library entry
    rp, col, val = W.out_row_ptr, W.out_col, W.out_val.view(np.float16).astype(np.float32)
    for n in range(N):
        for j in range(rp[n], rp[n + 1]):
            dense[n, col[j]] = np.float32(dense[n, col[j]]) + np.float32(val[j])   # both exact in fp16, the sum in fp32
    for k0 in range(0, K, M):
        Mc = min(M, K - k0)
        if Mc <= 16:
            break                                                               # the last chunk would take another kernel
        x = np.zeros((Mc, K), np.float16)
        x[np.arange(Mc), k0 + np.arange(Mc)] = 1.0
        y = xfp.xfp_gemv(dW, dev_x(x.view(np.uint16)), y_dtype=torch.float32)
        torch.cuda.synchronize()
        got = y.cpu().numpy()                                                   # [Mc][N]
        assert np.array_equal(got, dense[:, k0:k0 + Mc].T), (k0, np.argwhere(got != dense[:, k0:k0 + Mc].T)[:4])


def test_wide_kernel_bf16_activations_equal_the_converted_call():
    W = xi.random_weights(V2, 4, 64, 2048, density=0.003, seed=12)
    x = torch.randn(50, W.K, device="cuda")
    dW = xfp.upload(W)
    y_bf = xfp.xfp_gemv(dW, x.bfloat16(), y_dtype=torch.float32)
    y_h = xfp.xfp_gemv(dW, xfp.xfp_convert_bf16_to_f16(x.bfloat16()), y_dtype=torch.float32)
    assert torch.equal(y_bf, y_h)


def test_wide_kernel_bf16_output_is_one_rounding_of_the_fp32_result():
    W = xi.random_weights(V2, 4, 90, 2048, density=0.003, seed=15)
    dW = xfp.upload(W)
    xd = dev_x(xi.activations(np.random.default_rng(16), 37, W.K))
    y32 = xfp.xfp_gemv(dW, xd, y_dtype=torch.float32)
    ybf = xfp.xfp_gemv(dW, xd, y_dtype=torch.bfloat16)
    y16 = xfp.xfp_gemv(dW, xd, y_dtype=torch.float16)
    assert torch.equal(ybf, y32.bfloat16()) and torch.equal(y16, y32.half())


def test_strided_tokens_and_outputs():
    W = xi.random_weights(V2, 4, 100, 1024, density=0.003, seed=5)
    xb = xi.activations(np.random.default_rng(6), 30, 2 * W.K)                  # token rows of 2 K halves: stride 2 K
    xd = dev_x(xb)[:, :W.K]
    ybuf = torch.full((30, 128), 7.0, dtype=torch.float32, device="cuda")
    dW = xfp.upload(W)
    xfp.xfp_gemv(dW, xd, y=ybuf[:, :100])
    got = host(ybuf)
    ref = oracle.gemv_weights(W, np.ascontiguousarray(xb[:, :W.K]))
    assert gated_rel_err(got[:, :100], ref) <= 1e-4
    assert np.all(got[:, 100:] == 7.0)                                          # nothing written past N


def test_workload_5_shape_at_3_bits_with_48_tokens_full_size():
    """28672 x 8192, 3 bits (the matrix of bench.py --config 9), 48 tokens in one pass."""
    W = xi.random_weights(V2, 3, 28672, 8192, density=0.003, seed=xi.BASE_SEED + 9)
    check(W, xi.activations(np.random.default_rng(xi.BASE_SEED + 448), 48, W.K))


def test_library_matrix_of_configuration_10_with_64_tokens_full_size():
    """28672 x 8192, V2a 3-bit, L = 32 (the matrix of bench.py --config 10), 64 tokens in one pass."""
    W = xi.random_weights(V2A, 3, 28672, 8192, L=32, density=0.003, seed=xi.BASE_SEED + 10)
    check(W, xi.activations(np.random.default_rng(xi.BASE_SEED + 464), 64, W.K))


def test_workload_5_matrix_with_64_tokens_full_size():
    """28672 x 8192, 4 bits, 64 tokens in one pass: the size the timing in the design notes is quoted on."""
    W = xi.config_weights(5)
    x = xi.config_x(5, 64, W.K)
    check(W, x)


def test_long_rows_of_a_tall_matrix_take_one_launch_whatever_the_partial_planes_would_need():
    """16640 x 28672 with 3 tokens: the 16-token kernel would need four slices whose partial sums (4 x 16 x N
    floats) exceed its scratch plane; the wide kernel takes the rows whole, also through the entry point that
    allocates nothing (which refuses calls that only a larger plane would serve)."""
    W = xi.random_weights(V2, 4, 16640, 28672, density=0.001, seed=31)
    x = xi.activations(np.random.default_rng(32), 3, W.K)
    dW, xd, ref, y32 = check(W, x)
    assert xfp.xfp_route(dW, 3) == (xfp.XFP_ROUTE_WIDE, 3)
    y = torch.empty((3, W.N), dtype=torch.float32, device="cuda")
    xfp.xfp_gemv_noalloc(dW, xd, y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64), y32)


@pytest.mark.parametrize("mode,bits", [(V2, 4), (V2A, 3)])
def test_every_token_count_up_to_130(mode, bits):
    """Chunking: 64 + 64 + 2, 64 + 17, 64 + 1, 48 + ... whatever the count, every token's row must be the single-call
    row of that token (to rounding) and match the oracle."""
    W = xi.random_weights(mode, bits, 40, 1024, density=0.003, seed=77 + bits)
    x = xi.activations(np.random.default_rng(5), 130, W.K)
    dW, xd = xfp.upload(W), dev_x(x)
    ref = oracle.gemv_weights(W, x)
    for M in list(range(1, 70)) + [79, 80, 81, 96, 97, 113, 128, 129, 130]:
        y = host(xfp.xfp_gemv(dW, xd[:M].contiguous(), y_dtype=torch.float32))
        assert y.shape == (M, W.N)
        assert gated_rel_err(y, ref[:M]) <= 1e-4, M


@pytest.mark.parametrize("bits,N,K,M,L", [(3, 4096, 4096, 16, 32), (4, 2100, 8192, 9, 32), (2, 1030, 16384, 16, 7), (4, 33000, 512, 16, 63),
                                          (3, 600, 28672, 8, 200), (4, 8200, 4096, 35, 1)])
def test_scale_and_mid_point_per_group_with_several_tokens(bits, N, K, M, L):
    """Flagged V2a tensors with 2 .. 16 tokens per launch on the wide kernel (from 2^27 weights x tokens on): ragged
    last tile, rows of 4 and of 224 groups, more than 16 tokens in chunks; against the oracle, and every token's row
    against the single-token call (the streaming kernel's mode for the same tensors)."""
    W = xi.random_weights(V2A, bits, N, K, L=L, density=0.002, seed=N + K + bits, affine=True)
    x = xi.activations(np.random.default_rng(N + M), M, K)
    dW, xd = xfp.upload(W), dev_x(x)
    assert xfp.xfp_route(dW, M) == (xfp.XFP_ROUTE_WIDE, min(M, 16))
    ref = oracle.gemv_weights(W, x)
    y32 = host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float32))
    assert gated_rel_err(y32, ref) <= 1e-4
    assert gated_rel_err(host(xfp.xfp_gemv(dW, xd, y_dtype=torch.float16)), ref) <= 1e-3
    for m in (0, M - 1):
        y1 = host(xfp.xfp_gemv(dW, xd[m:m + 1].contiguous(), y_dtype=torch.float32))
        assert gated_rel_err(y32[m], y1[0]) <= 1e-4
    xb = xd.float().bfloat16()                                                  # bf16 activations: the converted call's bits
    assert torch.equal(xfp.xfp_gemv(dW, xb, y_dtype=torch.float32),
                       xfp.xfp_gemv(dW, xfp.xfp_convert_bf16_to_f16(xb), y_dtype=torch.float32))


def test_scale_and_mid_point_one_hot_is_the_affine_value():
    """One-hot tokens through the wide kernel's mode: y[m][n] = entry * scale + mid of one weight, one fp32 rounding
    of an exact product plus the mid-point (the block of the group holds the entry alone, the token's sum is 1)."""
    W = xi.random_weights(V2A, 4, 8200, 1024, L=9, density=0.0, seed=10, affine=True)
    dW = xfp.upload(W)
    q = oracle.unpack(W.indices[0], W.K, 4).astype(np.int64)
    lib = W.codebooks[0].view(np.float16).astype(np.float32)
    ids = np.repeat(W.group_ids[0].astype(np.int64), 128, axis=1)
    sc = np.repeat(W.group_scale[0].view(np.float16).astype(np.float32), 128, axis=1)
    md = np.repeat(W.group_mid[0].view(np.float16).astype(np.float32), 128, axis=1)
    want = (lib[ids, q].astype(np.float64) * sc.astype(np.float64) + md.astype(np.float64)).astype(np.float32)   # one rounding
    for k0 in (0, 500, 1008):
        x = np.zeros((16, W.K), np.float16)
        x[np.arange(16), k0 + np.arange(16)] = 1.0
        assert xfp.xfp_route(dW, 16)[0] == xfp.XFP_ROUTE_WIDE
        got = xfp.xfp_gemv(dW, dev_x(x.view(np.uint16)), y_dtype=torch.float32).cpu().numpy()
        assert np.array_equal(got, want[:, k0:k0 + 16].T)
