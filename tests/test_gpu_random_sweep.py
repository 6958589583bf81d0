"""Seeded random walk over what the dispatcher can be asked: format (V2 / V2a, 2 to 6 bits, with or without a scale
and a mid-point per group), shape (ragged row counts, group counts around every kernel's limits), token count,
outlier density, activation and output types, strides.  Every case goes through xfp_gemv and is compared with the
fp64 oracle on the same inputs; the route the call takes is printed so that a failure names its kernel."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_14844_amd as xfp
import xfp_inputs as xi
from helpers import gated_rel_err

pytestmark = pytest.mark.gpu
ROUTES = {getattr(xfp, n): n[10:] for n in dir(xfp) if n.startswith("XFP_ROUTE_")}
GROUPS = [1, 2, 3, 4, 5, 7, 8, 9, 11, 15, 16, 17, 23, 31, 32, 33, 40, 57, 64, 65, 96, 127, 128, 129, 136, 200, 256]
TOKENS = [1, 1, 1, 2, 3, 5, 8, 15, 16, 17, 18, 31, 32, 33, 40, 47, 48, 49, 63, 64, 65, 70, 81]


def draw(rng):
    mode = int(rng.integers(0, 2))
    bits = int(rng.choice([2, 3, 4, 4, 3, 2, 5, 6])) if mode == xi.MODE_V2 else int(rng.choice([2, 3, 4]))
    affine = mode == xi.MODE_V2A and rng.random() < 0.15
    G = int(rng.choice(GROUPS))
    M = int(rng.choice(TOKENS))
    if bits > 4 or affine:                                  # the general kernel goes token by token: keep it short
        G, M = min(G, 40), min(M, 5)
    N = int(rng.choice([1, 7, 16, 31, 32, 33, 63, 64, 65, 100, 129, 257]))
    while N * G * 128 * M > 3e8:                             # the oracle's work per case
        N = max(1, N // 2)
    L = int(rng.choice([1, 3, 32, 64])) if mode == xi.MODE_V2A else 32
    dens = float(rng.choice([0.0, 0.001, 0.003, 0.02]))
    return dict(mode=mode, bits=bits, affine=bool(affine), N=N, K=128 * G, M=M, L=L, dens=dens,
                x_bf16=bool(rng.random() < 0.25), y=str(rng.choice(["f32", "f16", "bf16"])),
                strided=bool(rng.random() < 0.2))


CASES = [draw(np.random.default_rng([2605, 14844, i])) for i in range(150)]
# long 4-bit rows with one token per call (the tile kernel) and long rows of the other widths (split-K) are rare
# in the draw above: ten cases of their own
for i, (bits, G, N) in enumerate([(4, 129, 33), (4, 200, 64), (4, 256, 7), (4, 131, 100), (4, 255, 32),
                                  (3, 136, 31), (2, 256, 16), (3, 255, 65), (2, 129, 129), (4, 224, 1)]):
    CASES.append(dict(draw(np.random.default_rng([2605, 14844, 150 + i])), mode=xi.MODE_V2, bits=bits, affine=False,
                      N=N, K=128 * G, M=1))


@pytest.mark.parametrize("chunk", range(8))
def test_random_calls_match_the_oracle(chunk):
    for idx in range(chunk * 20, chunk * 20 + 20):
        c = CASES[idx]
        W = xi.random_weights(c["mode"], c["bits"], c["N"], c["K"], L=c["L"], density=c["dens"], seed=7000 + idx,
                              affine=c["affine"])
        dW = xfp.upload(W)
        route = ROUTES[xfp.xfp_route(dW, c["M"])[0]]
        print(f"case {idx}: {c} -> {route}", flush=True)
        ldx = c["K"] + (64 if c["strided"] else 0)
        if c["x_bf16"]:
            # bf16 values in fp16's normal range convert exactly: the oracle gets the same numbers as fp16 bits
            xf = torch.randn(c["M"], ldx, generator=torch.Generator().manual_seed(idx)).clamp_(-8, 8)
            xf = torch.where(xf.abs() < 2.0 ** -10, torch.full_like(xf, 0.5), xf).bfloat16()
            x_bits = xf[:, :c["K"]].half().contiguous().view(torch.int16).numpy().view(np.uint16)
            xd = xf.cuda()[:, :c["K"]]
        else:
            full = xi.activations(np.random.default_rng(idx), c["M"], ldx)
            x_bits = np.ascontiguousarray(full[:, :c["K"]])
            xd = torch.from_numpy(full.view(np.int16)).cuda().view(torch.float16)[:, :c["K"]]
        ydt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[c["y"]]
        ldy = c["N"] + (24 if c["strided"] else 0)
        ybuf = torch.full((c["M"], ldy), -3.0, dtype=ydt, device="cuda")
        xfp.xfp_gemv(dW, xd, y=ybuf[:, :c["N"]])
        torch.cuda.synchronize()
        got = ybuf.float().cpu().numpy().astype(np.float64)
        ref = oracle.gemv_weights(W, x_bits)
        err = gated_rel_err(got[:, :c["N"]], ref)
        # one rounding of the output type on top of the fp32 bar: fp16 2^-11, bf16 2^-8
        tol = {"f32": 1e-4, "f16": 1e-3, "bf16": 6e-3}[c["y"]]
        assert err <= tol, (idx, c, route, err)
        assert np.all(got[:, c["N"]:] == -3.0), (idx, c, route)                 # nothing written past N
