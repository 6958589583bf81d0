"""Host-side checks that need no GPU: the library loads, exports what the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2605_14844_amd as xfp
from paper_2605_14844_amd.binding import xfp_weights

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a non-NULL, 16-byte aligned "device pointer" that is never dereferenced


def declared_functions():
    text = open(os.path.join(ROOT, "include", "xfp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(xfp_[a-z0-9_]+)\s*\(", text)))


def desc(**kw):
    d = xfp_weights()
    d.struct_size = ctypes.sizeof(xfp_weights)
    d.mode, d.bits, d.group, d.N, d.K, d.L, d.E = 0, 4, 128, 64, 256, 0, 1
    d.indices = d.codebooks = d.out_row_ptr = d.out_col = d.out_val = FAKE
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def gemv(d, x=FAKE, M=1, ldx=256, y=FAKE, dt=0, ldy=64):
    return xfp.load_library().xfp_gemv(ctypes.byref(d), x, M, ldx, y, dt, ldy, None)


def moe(d, ids=FAKE, T=2, x=FAKE, xs=0, y=FAKE, dt=0, ldy=64):
    return xfp.load_library().xfp_gemv_moe(ctypes.byref(d), ids, T, x, xs, y, dt, ldy, None)


def test_library_exports_every_declared_symbol():
    lib = xfp.load_library()
    names = declared_functions()
    assert {"xfp_gemv", "xfp_gemv_moe", "xfp_gemv_moe_silu_mul", "xfp_gemv_moe_combine", "xfp_check_contents", "xfp_convert_bf16_to_f16", "xfp_repack_word10", "xfp_unpack_indices", "xfp_dequant_bulk", "xfp_strerror",
            "xfp_version", "xfp_probe_read", "xfp_probe_copy"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert xfp.xfp_version() >= 0x100
    assert ctypes.sizeof(xfp_weights) == 104


def test_strerror_texts():
    assert xfp.xfp_strerror(0) == "ok"
    for s in (-1, -2, -3, -4):
        assert xfp.xfp_strerror(s) not in ("ok", "unknown status")
    assert xfp.xfp_strerror(-99) == "unknown status"


def test_null_pointers():
    assert xfp.load_library().xfp_gemv(None, FAKE, 1, 256, FAKE, 0, 64, None) == -1
    assert gemv(desc(indices=None)) == -1
    assert gemv(desc(codebooks=None)) == -1
    assert gemv(desc(out_row_ptr=None)) == -1
    assert gemv(desc(), x=None) == -1
    assert gemv(desc(), y=None) == -1
    assert gemv(desc(mode=1, L=32)) == -1                     # V2a without group ids
    assert moe(desc(E=4), ids=None) == -1
    lib = xfp.load_library()
    assert lib.xfp_unpack_indices(ctypes.byref(desc()), None, None) == -1
    assert lib.xfp_dequant_bulk(ctypes.byref(desc()), None, None) == -1


def test_shape_errors():
    assert gemv(desc(K=200)) == -2                             # K % 128
    assert gemv(desc(N=0)) == -2
    assert gemv(desc(K=0)) == -2
    assert gemv(desc(), M=0) == -2
    assert gemv(desc(), M=-3) == -2
    assert gemv(desc(), ldx=128) == -2                         # ldx < K
    assert gemv(desc(), ldy=10) == -2                          # ldy < N
    assert gemv(desc(E=2)) == -2                               # xfp_gemv takes one matrix
    assert moe(desc(E=4), T=-1) == -2
    assert moe(desc(E=4), xs=64) == -2                         # 0 < stride < K


def test_unsupported_format():
    for bits in (0, 1, 7, 8):
        assert gemv(desc(bits=bits)) == -3
    assert gemv(desc(mode=2)) == -3
    assert gemv(desc(group=64)) == -3
    assert gemv(desc(flags=1)) == -3                           # a scale and mid-point per group: V2a only
    assert gemv(desc(flags=2)) == -3 and gemv(desc(mode=1, L=32, group_ids=FAKE, flags=3, group_scale=FAKE, group_mid=FAKE)) == -3
    assert gemv(desc(mode=1, L=32, group_ids=FAKE, flags=1)) == -1                      # announced but not given
    assert gemv(desc(mode=1, L=32, group_ids=FAKE, flags=1, group_scale=FAKE)) == -1
    assert gemv(desc(mode=1, L=32, group_ids=FAKE, group_scale=FAKE, group_mid=FAKE)) == -3   # given but not announced
    assert gemv(desc(mode=1, L=32, group_ids=FAKE, flags=1, group_scale=FAKE + 1, group_mid=FAKE)) == -4
    assert gemv(desc(struct_size=80)) == -3
    assert gemv(desc(mode=1, L=0, group_ids=FAKE)) == -3
    assert gemv(desc(mode=1, L=300, group_ids=FAKE)) == -3
    assert gemv(desc(L=32)) == -3                              # L given for V2
    assert gemv(desc(), dt=3) == -3                            # bad y dtype (0 fp16, 1 fp32, 2 bf16)
    assert gemv(desc(), dt=0x200) == -3                        # unknown flag (0x100: x is bf16)


def test_rows_no_kernel_can_take_are_rejected_up_front():
    """Longer than the streaming kernel holds, no split into equal slices (a prime number of groups),
    and too long for the general kernel to stage in LDS: refused before anything is launched."""
    assert gemv(desc(K=128 * 1009, bits=3), ldx=128 * 1009) == -3
    assert gemv(desc(K=128 * 1009, bits=2), ldx=128 * 1009) == -3
    assert moe(desc(E=4, K=128 * 1009, bits=3), xs=128 * 1009) == -3
    # the same row at 4 bits (V2) is the tile kernel's, which takes any number of groups
    assert xfp.xfp_route(desc(K=128 * 1009), 1) == (xfp.XFP_ROUTE_TILE, 1)
    assert "too long" in xfp.xfp_strerror(-3) and "bf16" in xfp.xfp_strerror(-3)


def test_ring_slot_arithmetic():
    """Eager calls cycle through slots 0..3, calls recorded into a graph through 4..7; the two never meet,
    and a call takes one slot however many planes it uses (the ticket counter advances once per call)."""
    lib = xfp.load_library()
    lib.xfp_ring_slot.argtypes = [ctypes.c_uint, ctypes.c_int]
    eager = [lib.xfp_ring_slot(t, 0) for t in range(16)]
    rec = [lib.xfp_ring_slot(t, 1) for t in range(16)]
    assert eager == [0, 1, 2, 3] * 4 and rec == [4, 5, 6, 7] * 4
    assert lib.xfp_ring_slot(0xFFFFFFFF, 0) == 3 and lib.xfp_ring_slot(0xFFFFFFFF, 1) == 7     # wrap-around stays in range
    assert not set(eager) & set(rec)


def test_noalloc_entry_point_refuses_what_its_static_array_cannot_hold():
    """Checked on the host before anything is launched (the pointers are fakes)."""
    lib = xfp.load_library()
    call = lambda d, M, ldx: lib.xfp_gemv_noalloc(ctypes.byref(d), FAKE, M, ldx, FAKE, 0, d.N, None)
    assert call(desc(K=65536, bits=2), 2, 65536) == -6             # M >= 2: the re-laid activations hold K <= 32768
    assert call(desc(K=32768, N=300000, bits=3), 1, 32768) == -6   # M = 1 split-K (3 bits): 4 * N floats of partial sums > 2^20
    assert "scratch" in xfp.xfp_strerror(-6)
    assert call(desc(K=200), 1, 256) == -2 and call(desc(bits=9), 1, 256) == -3      # the usual validation comes first
    assert call(desc(E=2), 1, 256) == -2


def test_kernel_selection_takes_only_its_three_values():
    lib = xfp.load_library()
    assert lib.xfp_select_kernel(2) == 0 and lib.xfp_select_kernel(1) == 0 and lib.xfp_select_kernel(0) == 0
    assert lib.xfp_select_kernel(3) == -3 and lib.xfp_select_kernel(-1) == -3


def test_alignment_errors():
    assert gemv(desc(indices=FAKE + 4)) == -4
    assert gemv(desc(codebooks=FAKE + 2)) == -4
    assert gemv(desc(out_row_ptr=FAKE + 2)) == -4
    assert gemv(desc(), x=FAKE + 2) == -4
    assert gemv(desc(), y=FAKE + 8) == -4
    assert gemv(desc(), M=2, ldx=260) == -4
    assert moe(desc(E=4), xs=260) == -4


def test_moe_zero_slots_is_a_no_op():
    assert moe(desc(E=4), T=0, ids=None, x=None, y=None) == 0


def test_binding_rejects_bad_y_dtype_without_touching_the_gpu():
    import torch
    with pytest.raises(xfp.XfpError):
        xfp.binding._y_code(torch.float64)
    with pytest.raises(xfp.XfpError):
        xfp.binding._y_code(torch.float16, torch.zeros(4, dtype=torch.float32))     # x must be fp16 or bf16
    assert xfp.binding._y_code(torch.bfloat16) == xfp.XFP_BF16
    assert xfp.binding._y_code(torch.float32, torch.zeros(4, dtype=torch.bfloat16)) == xfp.XFP_F32 | xfp.XFP_X_BF16


def test_new_entry_points_reject_bad_arguments():
    """Every call below fails validation, so nothing is launched (the pointers are fakes)."""
    lib = xfp.load_library()
    d = desc(E=4)
    silu = lambda dd=d, ids=FAKE, T=2, x=FAKE, xs=0, h=FAKE, dt=0, ldh=32: lib.xfp_gemv_moe_silu_mul(
        ctypes.byref(dd), ids, T, x, xs, h, dt, ldh, None)
    assert silu(dd=desc(E=4, N=63)) == -2                      # N must be even
    assert silu(ldh=31) == -2                                  # ldh < N / 2
    assert silu(ids=None) == -1                                # ids required for a bank of several matrices
    assert silu(h=None) == -1 and silu(x=None) == -1
    assert silu(dt=7) == -3
    assert silu(T=0, ids=None, x=None, h=None) == 0
    comb = lambda ids=FAKE, T=2, x=FAKE, xs=256, w=FAKE, y=FAKE, dt=0: lib.xfp_gemv_moe_combine(
        ctypes.byref(d), ids, T, x, xs, w, y, dt, None)
    assert comb(T=0) == -2 and comb(xs=64) == -2
    assert comb(w=None) == -1 and comb(ids=None) == -1 and comb(y=None) == -1
    assert comb(w=FAKE + 2) == -4 and comb(dt=9) == -3
    cvt = lambda src=FAKE, ld=256, dst=FAKE, rows=2, cols=256: lib.xfp_convert_bf16_to_f16(src, ld, dst, rows, cols, None)
    assert cvt(src=None) == -1 and cvt(dst=None) == -1
    assert cvt(cols=100) == -2 and cvt(ld=128) == -2 and cvt(rows=-1) == -2
    assert cvt(src=FAKE + 2) == -4 and cvt(ld=260) == -4
    assert cvt(rows=0) == 0
    rpw = lambda src=FAKE, rows=4, K=256, bits=5, dst=FAKE: lib.xfp_repack_words(src, rows, K, bits, dst, None)
    assert rpw(bits=7) == -3 and rpw(bits=1) == -3 and rpw(src=None) == -1 and rpw(K=100) == -2 and rpw(rows=0) == 0
    assert rpw(src=FAKE + 2, bits=6) == -4 and rpw(src=FAKE + 1, bits=5) == -4
    rpk = lambda src=FAKE, rows=4, K=256, dst=FAKE: lib.xfp_repack_word10(src, rows, K, dst, None)
    assert rpk(src=None) == -1 and rpk(dst=None) == -1
    assert rpk(K=100) == -2 and rpk(K=0) == -2 and rpk(rows=-1) == -2 and rpk(rows=1 << 40) == -2
    assert rpk(src=FAKE + 2) == -4 and rpk(dst=FAKE + 1) == -4
    assert rpk(rows=0) == 0
    chk = lambda dd=d, cap=10, ids=None, T=0, rep=FAKE: lib.xfp_check_contents(ctypes.byref(dd), cap, ids, T, rep, None)
    assert chk(rep=None) == -1 and chk(cap=-1) == -2 and chk(rep=FAKE + 4) == -4
    assert chk(dd=desc(out_col=None)) == -1                   # entries claimed but no column array


def route(d, M, moe=False):
    return xfp.xfp_route(d, M, moe)


def test_dispatch_rule_on_the_host():
    """xfp_route reports the rule the decode calls execute (one function in the library serves both): the five
    workloads and the configurations bench.py times land on the kernels the design notes name, and the size
    limits sit where the header says."""
    R = xfp
    v2a = dict(mode=1, L=32, group_ids=FAKE)
    # the five workloads
    assert route(desc(N=512, K=1024), 1) == (R.XFP_ROUTE_STREAM, 1)                       # C1
    assert route(desc(N=8192, K=4096), 1) == (R.XFP_ROUTE_STREAM, 1)                      # C2: 2^25 weights
    assert route(desc(N=4096, K=4096, bits=3, **v2a), 1) == (R.XFP_ROUTE_STREAM, 1)       # C3
    assert route(desc(N=2048, K=4096, bits=3, E=256), 8, moe=True) == (R.XFP_ROUTE_STREAM, 8)   # C4 gate_up
    assert route(desc(N=28672, K=8192), 16) == (R.XFP_ROUTE_BATCH, 16)                    # C5
    # M = 1: the tile kernel from 2^26 weights per call on and for rows beyond 16384 columns (4-bit V2 only)
    assert route(desc(N=16384, K=4096), 1) == (R.XFP_ROUTE_TILE, 1)
    assert route(desc(N=8192, K=28672), 1) == (R.XFP_ROUTE_TILE, 1)
    # 2 .. 16 tokens on rows the 16-token kernel would cut into slices: the wide kernel once its tiles fill the chip
    assert route(desc(N=8192, K=28672), 16) == (R.XFP_ROUTE_WIDE, 16)
    assert route(desc(N=8192, K=28672, bits=3), 5) == (R.XFP_ROUTE_WIDE, 5)
    assert route(desc(N=8160, K=28672), 16) == (R.XFP_ROUTE_BATCH, 16)
    assert route(desc(N=4096, K=16384), 16) == (R.XFP_ROUTE_BATCH, 16)
    assert route(desc(N=64, K=16384 + 128), 1) == (R.XFP_ROUTE_TILE, 1)
    assert route(desc(N=16384, K=4096, bits=3), 1) == (R.XFP_ROUTE_STREAM, 1)
    assert route(desc(N=8192, K=28672, bits=3), 1) == (R.XFP_ROUTE_SPLIT_K, 1)
    assert route(desc(N=2048, K=4096, E=16), 8, moe=True) == (R.XFP_ROUTE_TILE, 8)        # 8 slots x 2^23 weights
    # tokens: 2 .. 16 the batched kernel; more: as many as the wide kernel's copies hold, then the rest
    assert route(desc(N=64, K=8192), 2) == (R.XFP_ROUTE_BATCH, 2)
    assert route(desc(N=64, K=8192), 17) == (R.XFP_ROUTE_WIDE, 17)
    assert route(desc(N=64, K=8192), 64) == (R.XFP_ROUTE_WIDE, 64)
    assert route(desc(N=64, K=8192), 200) == (R.XFP_ROUTE_WIDE, 64)
    assert route(desc(N=64, K=8192 + 128), 64) == (R.XFP_ROUTE_WIDE, 48)                  # 16 * 3 * K <= 2^19 < 16 * 4 * K
    assert route(desc(N=64, K=16384), 64) == (R.XFP_ROUTE_WIDE, 32)
    assert route(desc(N=64, K=16384 + 128), 64) == (R.XFP_ROUTE_BATCH, 16)                # one chunk only: chunks of 16
    assert route(desc(N=64, K=8192, bits=3), 40) == (R.XFP_ROUTE_WIDE, 40)
    assert route(desc(N=64, K=8192, bits=3, **v2a), 40) == (R.XFP_ROUTE_WIDE, 40)
    assert route(desc(N=64, K=8192, bits=2, **v2a), 40) == (R.XFP_ROUTE_WIDE, 40)
    # widths 5 and 6 and tensors with a scale and a mid-point per group: the general kernel, token by token
    assert route(desc(N=64, K=4096, bits=5), 3) == (R.XFP_ROUTE_GENERAL, 3)
    # a scale and a mid-point per group: the streaming kernel's own mode for rows it holds, token by token; else general
    assert route(desc(N=64, K=4096, flags=1, group_scale=FAKE, group_mid=FAKE, **v2a), 1) == (R.XFP_ROUTE_STREAM, 1)
    assert route(desc(N=64, K=4096, bits=3, flags=1, group_scale=FAKE, group_mid=FAKE, **v2a), 40) == (R.XFP_ROUTE_STREAM, 40)
    # ... and from 2^27 weights x tokens on through the wide kernel's mode for them, 16 tokens per launch
    assert route(desc(N=4096, K=4096, bits=3, flags=1, group_scale=FAKE, group_mid=FAKE, **v2a), 8) == (R.XFP_ROUTE_WIDE, 8)
    assert route(desc(N=4096, K=4096, bits=3, flags=1, group_scale=FAKE, group_mid=FAKE, **v2a), 4) == (R.XFP_ROUTE_STREAM, 4)
    assert route(desc(N=28672, K=8192, bits=3, flags=1, group_scale=FAKE, group_mid=FAKE, **v2a), 40) == (R.XFP_ROUTE_WIDE, 16)
    assert route(desc(N=28672, K=8192, bits=3, flags=1, group_scale=FAKE, group_mid=FAKE, **v2a), 1) == (R.XFP_ROUTE_STREAM, 1)
    assert route(desc(N=64, K=20480, flags=1, group_scale=FAKE, group_mid=FAKE, **v2a), 1) == (R.XFP_ROUTE_GENERAL, 1)
    # what xfp_select_kernel changes, xfp_route reports
    xfp.xfp_select_kernel(xfp.XFP_KERNEL_TILE)
    try:
        assert route(desc(N=512, K=1024), 1) == (R.XFP_ROUTE_TILE, 1)
    finally:
        xfp.xfp_select_kernel(xfp.XFP_KERNEL_AUTO)
    # errors come back as the decode calls would raise them
    with pytest.raises(xfp.XfpError) as ei:
        route(desc(K=128 * 1009, bits=3), 1)
    assert ei.value.status == -3
    with pytest.raises(xfp.XfpError):
        route(desc(K=200), 1)


def test_dispatch_invariants_over_random_descriptors():
    """Whatever the descriptor, every launch takes between 1 and the remaining tokens: 2 .. 16 on the batched route,
    2 .. 64 on the wide one, all of them on the M = 1 routes; and walking a call launch by launch terminates."""
    import random
    rnd = random.Random(2605)
    R = xfp
    names = {getattr(R, n) for n in dir(R) if n.startswith("XFP_ROUTE_")}
    for _ in range(3000):
        mode = rnd.choice([0, 0, 1])
        bits = rnd.choice([2, 3, 4, 5, 6]) if mode == 0 else rnd.choice([2, 3, 4])
        kw = dict(N=rnd.choice([1, 31, 32, 33, 4096, 8160, 8161, 8192, 28672, 70000]), K=128 * rnd.choice([1, 2, 7, 8, 63, 64, 65, 128, 129, 224, 256, 257, 512]),
                  bits=bits)
        if mode == 1:
            kw.update(mode=1, L=rnd.choice([1, 32, 64, 65, 256]), group_ids=FAKE)
        d = desc(**kw)
        M = rnd.choice([1, 2, 15, 16, 17, 33, 63, 64, 65, 200])
        left, launches = M, 0
        while left:
            try:
                r, n = xfp.xfp_route(d, left)
            except xfp.XfpError as e:
                assert e.status == -3                         # a row no kernel takes
                break
            assert r in names and 1 <= n <= left, (kw, M, left, r, n)
            if r == R.XFP_ROUTE_BATCH:
                assert 2 <= n <= 16, (kw, M, left, r, n)
            elif r == R.XFP_ROUTE_WIDE:
                assert 2 <= n <= 64, (kw, M, left, r, n)
            else:
                assert n == left, (kw, M, left, r, n)         # the M = 1 kernels take every remaining token as a slot
            left -= n
            launches += 1
            assert launches <= M
