"""The .xfp file round trip and the storage-size model against the paper's printed figures."""
import os

import numpy as np
import pytest

import xfp_inputs as xi
from paper_2605_14844_amd import bytes_per_weight, load_xfp, save_xfp

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_size_facts.txt")


def facts():
    out = {}
    for line in open(GOLDEN):
        t = line.split("#")[0].split()
        if t and t[0] != "pack":
            out[t[0]] = float(t[1])
    return out


@pytest.mark.parametrize("mode,bits,E,affine", [(xi.MODE_V2, 4, 1, False), (xi.MODE_V2A, 3, 1, False), (xi.MODE_V2, 3, 5, False),
                                                (xi.MODE_V2, 2, 1, False), (xi.MODE_V2, 5, 2, False), (xi.MODE_V2A, 6, 1, False),
                                                (xi.MODE_V2A, 4, 3, True)])
def test_save_load_bit_identical(tmp_path, mode, bits, E, affine):
    W = xi.random_weights(mode, bits, 48, 384, E=E, density=0.004, seed=3, affine=affine)
    p = str(tmp_path / "w.xfp")
    save_xfp(p, W)
    for mmap in (True, False):
        R = load_xfp(p, mmap=mmap)
        assert (R.mode, R.bits, R.N, R.K, R.L, R.E, R.group) == (W.mode, W.bits, W.N, W.K, W.L, W.E, 128)
        for name in ("indices", "codebooks", "group_ids", "out_row_ptr", "out_col", "out_val", "group_scale", "group_mid"):
            a, b = getattr(W, name), getattr(R, name)
            if a is None:
                assert b is None
            else:
                assert a.dtype == b.dtype and a.shape == b.shape and np.array_equal(a, b), name


def test_empty_outliers_and_bad_files(tmp_path):
    W = xi.random_weights(xi.MODE_V2, 4, 8, 128, density=0.0, seed=4)
    p = str(tmp_path / "e.xfp")
    save_xfp(p, W)
    R = load_xfp(p)
    assert R.out_col.shape == (0,) and R.out_row_ptr.tolist() == [0] * 9
    bad = tmp_path / "bad.xfp"
    bad.write_bytes(b"NOTANXFPFILE0000")
    with pytest.raises(ValueError):
        load_xfp(str(bad))


def test_size_model_reproduces_paper_figures():
    f = facts()
    coo = f["outlier_triple_bytes"]
    assert coo == 18
    assert bytes_per_weight(4, 0.02, coo) - bytes_per_weight(4, 0.0, coo) == pytest.approx(
        f["outlier_bytes_per_weight_at_cap"])
    # break-even of 3-bit with y outliers against 4-bit at the 2 % cap (indices + COO outliers only)
    lhs = lambda y: bytes_per_weight(3, y, coo)
    rhs = bytes_per_weight(4, 0.02, coo)
    y = (rhs - lhs(0.0)) / coo
    assert round(y, 3) == f["break_even_outlier_fraction"]
    assert lhs(y) == pytest.approx(rhs)
    # V2a: 32 codebooks of 16 fp16 entries = 1 KB; a 40-bit group record = 0.31 bit/weight
    assert 32 * 16 * 2 == f["v2a_library_bytes_n4_l32"]
    for n, key in ((2, "v2a_effective_bits_n2"), (4, "v2a_effective_bits_n4")):
        eff = 8 * bytes_per_weight(n, 0.0, mode=1, group_record_bits=40)
        assert round(eff, 2) == f[key]
    assert round(40 / 128, 2) == f["v2a_group_overhead_bits"]
