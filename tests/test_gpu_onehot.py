"""Bit-exact parity of the HOT kernels' own depack + codebook gather (paper section 5, steps 1 and 2).

With a one-hot activation row (1.0 at column k, zeros elsewhere) and fp32 output, every product but one is an
exact zero and the one is exact, so
    y[n] == fp32( C[n, k] + O[n, k] )
must hold with `==`, no tolerance (C: the codebook entry the index selects, O: the outlier at that position;
the fp64 sum of the two fp16 values rounded once to fp32 is what one fp32 addition gives).  Sweeping k over
EVERY column puts the whole dequantized matrix through the kernel that the decode calls really run: the
streaming kernel (every chunk count, short rows, tails, every batch size), its split-K and gate/up forms, the
combine kernel, and the batched matrix-core kernel (register transposition, bank-private tables, slices of K,
library tables).  A wrong pair in any lane, chunk, group or word-straddling field fails one comparison.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_14844_amd as xfp
import xfp_inputs as xi

pytestmark = pytest.mark.gpu
V2, V2A = xi.MODE_V2, xi.MODE_V2A


def expected_dense(W, e=0):
    """fp32( C + O ) of matrix e, [N, K], from the oracle's dequantized bits and the CSR arrays."""
    gid = None if W.group_ids is None else W.group_ids[e]
    bits16, _ = oracle.dequant_bulk(W.mode, W.bits, W.N, W.K, W.indices[e], W.codebooks[e], gid, want_double=False)
    d = bits16.view(np.float16).astype(np.float64)
    rp = W.out_row_ptr[e * W.N:(e + 1) * W.N + 1].astype(np.int64)
    rows = np.repeat(np.arange(W.N), np.diff(rp))
    sl = slice(rp[0], rp[-1])
    d[rows, W.out_col[sl]] += W.out_val[sl].view(np.float16).astype(np.float64)
    return d.astype(np.float32)


def one_hot_rows(k0, T, K, dtype=torch.float16):
    x = torch.zeros((T, K), dtype=dtype, device="cuda")
    r = torch.arange(T, device="cuda")
    x[r, k0 + r] = 1.0
    return x


def same(a, b):
    """Equality of values (+0 == -0), no NaNs expected."""
    return a.shape == b.shape and bool(np.all(a == b))


def special_codebook_entries(W):
    """Subnormal, zero, negative zero and extreme fp16 patterns among the entries."""
    cb = W.codebooks.reshape(-1, W.codebooks.shape[-1])
    cb[0, :4] = np.array([0x0001, 0x8000, 0x83FF, 0x7BFF], dtype=np.uint16)


# ------------------------------------------------------------------ streaming kernel, M = 1 per slot
# T: one-hot rows per launch.  The launcher's batch size U follows from N * T (one batch per wave up to 6144
# waves for V2, 3072 for V2a), so the T values below put U = 1, 2 and 4 of every shape through the sweep.
STREAM_SHAPES = [
    # mode, bits, N, K, density
    (V2, 4, 6, 512, 0.0), (V2, 4, 6, 1024, 0.004), (V2, 4, 5, 2048, 0.0), (V2, 4, 5, 4096, 0.003),
    (V2, 4, 3, 640, 0.0), (V2, 4, 3, 5120, 0.002), (V2, 4, 2, 8192, 0.0), (V2, 4, 2, 16384, 0.0),
    (V2, 3, 6, 512, 0.0), (V2, 3, 6, 1024, 0.004), (V2, 3, 5, 4096, 0.003), (V2, 3, 3, 2176, 0.0), (V2, 3, 2, 12288, 0.0),
    (V2, 2, 6, 512, 0.0), (V2, 2, 6, 1024, 0.0), (V2, 2, 5, 4096, 0.003), (V2, 2, 3, 1408, 0.0), (V2, 2, 2, 16384, 0.0),
    (V2A, 4, 5, 4096, 0.003), (V2A, 4, 3, 5120, 0.0), (V2A, 4, 6, 1024, 0.0), (V2A, 3, 5, 4096, 0.003),
    (V2A, 3, 3, 640, 0.0), (V2A, 3, 2, 8192, 0.0), (V2A, 2, 5, 2048, 0.0), (V2A, 2, 3, 896, 0.002),
]


@pytest.mark.parametrize("T", [256, 2048])
@pytest.mark.parametrize("mode,bits,N,K,dens", STREAM_SHAPES)
def test_streaming_kernel_one_hot_sweep(mode, bits, N, K, dens, T):
    W = xi.random_weights(mode, bits, N, K, density=dens, seed=7000 + bits * 100 + N + K)
    special_codebook_entries(W)
    dW = xfp.upload(W)
    want = expected_dense(W)
    ids = torch.zeros(T, dtype=torch.int32, device="cuda")
    for k0 in range(0, K, T):
        Tc = min(T, K - k0)
        y = xfp.xfp_gemv_moe(dW, ids[:Tc], one_hot_rows(k0, Tc, K), y_dtype=torch.float32)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert same(got, want[:, k0:k0 + Tc].T), (mode, bits, N, K, k0, np.argwhere(got != want[:, k0:k0 + Tc].T)[:5])


def test_streaming_kernel_one_hot_single_call_per_column():
    """The plain xfp_gemv M = 1 call (one slot, the batch size of a small launch), a call per column."""
    for mode, bits, N, K in ((V2, 4, 8, 1024), (V2, 3, 12, 640), (V2A, 4, 4, 2176)):
        W = xi.random_weights(mode, bits, N, K, density=0.003, seed=7100 + K)
        dW = xfp.upload(W)
        want = expected_dense(W)
        eye = one_hot_rows(0, K, K)
        Y = torch.empty((K, N), dtype=torch.float32, device="cuda")
        for k in range(K):
            xfp.xfp_gemv(dW, eye[k], y=Y[k])
        torch.cuda.synchronize()
        assert same(Y.cpu().numpy(), want.T)


# rows longer than the streaming kernel holds: split-K (slices of K, partial sums added in slice order)
@pytest.mark.parametrize("mode,bits,N,K", [(V2, 4, 3, 20480), (V2, 3, 2, 24576), (V2A, 3, 2, 32768), (V2, 2, 2, 28672),
                                           (V2A, 4, 2, 18432)])
def test_split_k_one_hot_sweep(mode, bits, N, K):
    W = xi.random_weights(mode, bits, N, K, density=0.001, seed=7200 + bits)
    dW = xfp.upload(W)
    want = expected_dense(W)
    T = 1024
    ids = torch.zeros(T, dtype=torch.int32, device="cuda")
    for k0 in range(0, K, T):
        y = xfp.xfp_gemv_moe(dW, ids, one_hot_rows(k0, T, K), y_dtype=torch.float32)
        torch.cuda.synchronize()
        assert same(y.cpu().numpy(), want[:, k0:k0 + T].T), (mode, bits, K, k0)


# ------------------------------------------------------------------ gate/up form (SiLU(gate) * up in the store)
@pytest.mark.parametrize("mode,bits,half,K", [(V2, 4, 4, 4096), (V2, 3, 4, 1024), (V2, 3, 3, 4096), (V2, 2, 2, 2048),
                                              (V2A, 3, 4, 2048), (V2, 4, 3, 640)])
def test_gate_up_form_one_hot_sweep(mode, bits, half, K):
    """h = SiLU(g) * u is not exact arithmetic, so each half is isolated in turn.
    Up rows: every gate entry is 1.0, so g == 1.0 for every column and h == s1 * u with ONE fp32 product, where
    s1 = SiLU(1.0) as the kernel computes it, read off an up position whose entry is 1.0: bit-exact.
    Gate rows: every up entry is 1.0, so h == SiLU(C[j, k]) * 1; adjacent fp16 entries differ by >= 2^-11
    relative, SiLU is smooth, so agreement to 2e-6 relative with the oracle's SiLU pins the entry that was read."""
    N = 2 * half
    one = np.uint16(0x3C00)
    for which in ("up", "gate"):
        W = xi.random_weights(mode, bits, N, K, density=0.0, seed=7300 + K + bits)
        cb = W.codebooks[0]
        if mode == V2:
            if which == "up":
                cb[:half, :] = one
                cb[half, oracle.unpack(W.indices[0], K, bits)[half, 0]] = one    # a known 1.0: up row 0, column 0
            else:
                cb[half:, :] = one
        else:
            # a library is shared by gate and up rows: entries 0..ENT/2-1 of every codebook random, the upper
            # half 1.0; the gate (or up) rows only use upper-half indices, the others only lower-half ones
            ent = 1 << bits
            cb[:, ent // 2:] = one
            q = oracle.unpack(W.indices[0], K, bits)
            fixed = slice(0, half) if which == "up" else slice(half, N)
            free = slice(half, N) if which == "up" else slice(0, half)
            q[fixed] |= ent // 2
            q[free] &= ent // 2 - 1
            if which == "up":
                q[half, 0] |= ent // 2
            W.indices[0] = xi.pack_bitstream(q, bits)
        dW = xfp.upload(W)
        C = expected_dense(W)                                  # density 0: the codebook values
        T = min(K, 512)
        ids = torch.zeros(T, dtype=torch.int32, device="cuda")
        H = np.empty((K, half), dtype=np.float32)
        for k0 in range(0, K, T):
            Tc = min(T, K - k0)
            h = xfp.xfp_gemv_moe_silu_mul(dW, ids[:Tc], one_hot_rows(k0, Tc, K), h_dtype=torch.float32)
            torch.cuda.synchronize()
            H[k0:k0 + Tc] = h.cpu().numpy()
        if which == "up":
            assert C[half, 0] == 1.0
            s1 = H[0, 0]                                       # SiLU(1.0) * 1.0 as the kernel computes it
            assert abs(float(s1) - 0.7310585786300049) < 1e-6
            assert same(H, (np.float32(s1) * C[half:, :]).T.astype(np.float32))
        else:
            g = C[:half, :].T.astype(np.float64)
            ref = oracle.silu_mul(np.concatenate([g, np.ones_like(g)], axis=1))
            assert np.all(np.abs(H - ref) <= 2e-6 * np.abs(ref) + 1e-30), np.max(np.abs(H - ref) / (np.abs(ref) + 1e-30))


# ------------------------------------------------------------------ combine kernel (weighted sum over slots)
@pytest.mark.parametrize("bits,N,K,E,T", [(3, 4, 1024, 5, 8), (4, 4, 640, 3, 5), (2, 4, 512, 4, 8), (4, 4, 2048, 9, 8),
                                          (3, 8, 384, 2, 7), (4, 4, 1024, 6, 2)])
def test_combine_kernel_one_hot_sweep(bits, N, K, E, T):
    """One-hot router weights and one one-hot activation row per slot: slot t0 of the call reads column k of its
    expert, every other slot is multiplied by an exact zero.  Each call checks column k of T different
    (slot, expert) pairs at once by giving every slot its OWN one-hot weight in turn."""
    W = xi.random_weights(V2, bits, N, K, E=E, density=0.002, seed=7400 + bits + K)
    dW = xfp.upload(W)
    want = [expected_dense(W, e) for e in range(E)]
    rng = np.random.default_rng(7400 + K)
    ids = rng.integers(0, E, size=T).astype(np.int32)
    ids_d = torch.from_numpy(ids).cuda()
    eye_w = torch.eye(T, dtype=torch.float32, device="cuda")
    step = 1 if K <= 640 else 3                                # every column of short rows, every third beyond
    cols = list(range(0, K, step)) + [K - 1]
    Y = torch.empty((len(cols), T, N), dtype=torch.float32, device="cuda")
    for ci, k in enumerate(cols):
        x = torch.zeros((T, K), dtype=torch.float16, device="cuda")
        x[:, k] = 1.0
        for t0 in range(T):
            xfp.xfp_gemv_moe_combine(dW, ids_d, x, eye_w[t0], y=Y[ci, t0])
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    for ci, k in enumerate(cols):
        for t0 in range(T):
            assert same(got[ci, t0], want[ids[t0]][:, k]), (bits, K, k, t0)


# ------------------------------------------------------------------ batched (matrix-core) kernel
@pytest.mark.parametrize("mode,bits,N,K,dens", [
    (V2, 4, 16, 1024, 0.0), (V2, 4, 37, 4096, 0.003), (V2, 4, 20, 8192, 0.0), (V2, 4, 17, 640, 0.002),
    (V2, 4, 18, 12288, 0.001), (V2, 4, 16, 28672, 0.0),
    (V2, 3, 33, 4096, 0.003), (V2, 3, 16, 1152, 0.0), (V2, 3, 18, 16384, 0.0),
    (V2, 2, 35, 2048, 0.003), (V2, 2, 16, 8192, 0.0), (V2, 2, 16, 9216, 0.0),
    (V2A, 3, 33, 4096, 0.003), (V2A, 3, 16, 10240, 0.0), (V2A, 4, 19, 2048, 0.002), (V2A, 4, 16, 8192, 0.0),
    (V2A, 2, 21, 2048, 0.003), (V2A, 2, 16, 12288, 0.0)])
def test_batched_kernel_one_hot_sweep(mode, bits, N, K, dens):
    """Every launch of the batched kernel takes 16 one-hot rows (16 different columns); the API walks the K rows
    of the identity in chunks of 16.  M = 5 and M = 2 launches cover the ragged token counts."""
    W = xi.random_weights(mode, bits, N, K, density=dens, seed=7500 + bits * 10 + N)
    special_codebook_entries(W)
    dW = xfp.upload(W)
    want = expected_dense(W)
    R = 2048                                                   # rows of the identity per call (128 launches)
    for k0 in range(0, K, R):
        y = xfp.xfp_gemv(dW, one_hot_rows(k0, min(R, K - k0), K), y_dtype=torch.float32)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert same(got, want[:, k0:k0 + R].T), (mode, bits, N, K, k0, np.argwhere(got != want[:, k0:k0 + R].T)[:5])
    for M, k0 in ((5, K - 5), (2, 64), (3, K // 2 + 29)):
        y = xfp.xfp_gemv(dW, one_hot_rows(k0, M, K), y_dtype=torch.float32)
        torch.cuda.synchronize()
        assert same(y.cpu().numpy(), want[:, k0:k0 + M].T), (mode, bits, N, K, M, k0)


# ------------------------------------------------------------------ general (fallback) kernel
@pytest.mark.parametrize("mode,bits,N,K", [(V2, 4, 5, 128 * 131), (V2, 3, 4, 128 * 137), (V2A, 2, 3, 128 * 139)])
def test_general_kernel_one_hot_sampled(mode, bits, N, K):
    """Rows longer than the streaming kernel with a prime number of groups (no split) run the general kernel."""
    W = xi.random_weights(mode, bits, N, K, density=0.001, seed=7600 + bits)
    dW = xfp.upload(W)
    want = expected_dense(W)
    T = 512
    ids = torch.zeros(T, dtype=torch.int32, device="cuda")
    for k0 in (0, 2048 - 256, K // 2, K - T):
        y = xfp.xfp_gemv_moe(dW, ids, one_hot_rows(k0, T, K), y_dtype=torch.float32)
        torch.cuda.synchronize()
        assert same(y.cpu().numpy(), want[:, k0:k0 + T].T), (mode, bits, K, k0)


# ------------------------------------------------------------------ bf16 activations, converted in the x load
@pytest.mark.parametrize("mode,bits,N,K,M", [(V2, 4, 40, 4096, 1), (V2, 3, 33, 1024, 1), (V2A, 3, 20, 5120, 1), (V2, 4, 24, 20480, 1),
                                             (V2, 4, 32, 4096, 16), (V2, 3, 20, 12288, 7), (V2A, 4, 18, 2048, 33),
                                             (V2, 2, 6, 128 * 131, 2)])
def test_bf16_activations_equal_the_call_on_the_converted_activations(mode, bits, N, K, M):
    """Every kernel converts bf16 activations as it loads them, with the arithmetic of xfp_convert_bf16_to_f16:
    the result must equal, bit for bit, the fp16 call on the converted tensor (values beyond fp16's range, tiny
    ones and an exact 0 included)."""
    W = xi.random_weights(mode, bits, N, K, density=0.003, seed=7700 + K)
    dW = xfp.upload(W)
    g = torch.Generator(device="cuda").manual_seed(7700 + K + M)
    xb = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    xb[0, 5], xb[0, 6], xb[0, 7], xb[0, 8] = 1e5, -3e38, 1e-7, 0.0
    # an outlier column gets an out-of-range value too (the gathers convert on their own)
    if W.nnz:
        xb[0, int(W.out_col[0])] = -7e4
    xh = xfp.xfp_convert_bf16_to_f16(xb)
    for dt in (torch.float32, torch.float16):
        a = xfp.xfp_gemv(dW, xb if M > 1 else xb[0], y_dtype=dt)
        b = xfp.xfp_gemv(dW, xh if M > 1 else xh[0], y_dtype=dt)
        torch.cuda.synchronize()
        assert torch.equal(a, b), (mode, bits, N, K, M, dt)
