"""xfp_gemv_noalloc (scratch in one static device array, nothing allocated) against xfp_gemv.

Both run the same kernels, so the outputs must be equal bit for bit, which is tighter than the parity bars
(1e-3 gated for fp16 y, 1e-4 for fp32 y); the oracle is checked beside it.  Every case makes two calls in a
row on the shared array, the second smaller than the first, so anything the first leaves behind in the
array would show in the second."""
import ctypes

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


def one_call(mode, bits, N, K, M, seed, dtype):
    W = xi.random_weights(mode, bits, N, K, density=0.003, seed=seed)
    xb = xi.activations(np.random.default_rng(seed + 1), M, K)
    dW, xd = xfp.upload(W), dev_x(xb)
    y = torch.empty((M, N), dtype=dtype, device="cuda")
    xfp.xfp_gemv_noalloc(dW, xd if M > 1 else xd[0], y)
    want = xfp.xfp_gemv(dW, xd if M > 1 else xd[0], y_dtype=dtype)
    torch.cuda.synchronize()
    assert torch.equal(y, want), (mode, bits, N, K, M)
    ref = oracle.gemv_weights(W, xb)
    assert gated_rel_err(y.float().cpu().numpy().astype(np.float64), ref) <= (1e-4 if dtype == torch.float32 else 1e-3)


@pytest.mark.parametrize("first,second", [
    # batched kernel over slices of K (re-laid activations + partial planes), then a smaller batched call
    ((V2, 4, 96, 12288, 16), (V2, 4, 40, 2048, 5)),
    # split-K of the M = 1 kernel (partial planes), then a shorter split
    ((V2, 3, 200, 24576, 1), (V2, 3, 64, 20480, 1)),
    # V2a batched, several chunks of 16 and an odd token; then M = 1 with no scratch at all
    ((V2A, 3, 70, 10240, 35), (V2A, 3, 33, 4096, 1)),
    ((V2, 2, 128, 32768, 4), (V2, 2, 16, 128, 2)),
    # more than 16 tokens in one pass over the weights (wider re-laid copies in the same array), then 16 tokens
    ((V2, 4, 100, 8192, 64), (V2, 4, 50, 4096, 16)),
    ((V2, 3, 77, 16384, 40), (V2, 3, 33, 1024, 20)),
    # the same for a library format (V2a), then 2-bit V2a on the 16-token kernel
    ((V2A, 3, 90, 8192, 64), (V2A, 2, 40, 2048, 9)),
])
def test_two_calls_in_a_row_match_xfp_gemv(first, second):
    for dtype in (torch.float32, torch.float16):
        one_call(*first, seed=9100, dtype=dtype)
        one_call(*second, seed=9200, dtype=dtype)


def test_sizes_beyond_the_static_array_are_refused():
    """Where xfp_gemv would take another route because a scratch plane is too small, this entry point says so."""
    W = xi.random_weights(V2, 2, 4, 65536, density=0.0, seed=9300)            # M >= 2 with K > 32768
    dW = xfp.upload(W)
    x = torch.zeros((2, W.K), dtype=torch.float16, device="cuda")
    y = torch.empty((2, W.N), dtype=torch.float32, device="cuda")
    with pytest.raises(xfp.XfpError) as ei:
        xfp.xfp_gemv_noalloc(dW, x, y)
    assert ei.value.status == -6 and "scratch" in str(ei.value)
    xfp.xfp_gemv(dW, x, y=y)                                                   # the ring-backed call reroutes instead
    torch.cuda.synchronize()


def test_flagged_tensor_with_several_tokens_matches_xfp_gemv():
    """A scale and a mid-point per group, 16 then 5 tokens: the wide kernel's mode for them keeps its activation sums
    in a scratch plane of the same static array."""
    for (N, M, seed) in ((2100, 16, 9400), (8300, 5, 9500)):
        W = xi.random_weights(V2A, 3, N, 4096, density=0.002, seed=seed, affine=True)
        xb = xi.activations(np.random.default_rng(seed + 1), M, W.K)
        dW, xd = xfp.upload(W), dev_x(xb)
        assert xfp.xfp_route(dW, M)[0] == xfp.XFP_ROUTE_WIDE
        y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        xfp.xfp_gemv_noalloc(dW, xd, y)
        want = xfp.xfp_gemv(dW, xd, y_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(y, want)
        assert gated_rel_err(y.cpu().numpy().astype(np.float64), oracle.gemv_weights(W, xb)) <= 1e-4
