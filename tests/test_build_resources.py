"""What the compiler made of the kernels (registers, spills, occupancy), read from the remarks the build keeps
in kernel_resources.json.  A change in front of a kernel's loads can silently cost it a wave per SIMD or push it
into scratch memory (a three-line branch once did: 35 registers, 98 spilled, a 2.4 times slower call), so the
kernels that the five workloads launch are pinned here."""
import json
import os

import pytest

import paper_2605_14844_amd as xfp

PATH = os.path.join(os.path.dirname(xfp.library_path()), "kernel_resources.json")


def resources():
    if not os.path.exists(PATH):
        pytest.skip("kernel_resources.json is written by paper_2605_14844_amd.build.build()")
    with open(PATH) as f:
        return json.load(f)


def find(res, *parts):
    hits = [v for k, v in res.items() if all(p in k for p in parts)]
    assert len(hits) == 1, (parts, len(hits))
    return hits[0]


def test_no_kernel_spills_more_than_a_few_registers():
    res = resources()
    assert len(res) > 500
    worst = max(res.items(), key=lambda kv: kv[1]["vgpr_spills"])
    assert worst[1]["vgpr_spills"] <= 16, worst
    assert sum(1 for v in res.values() if v["vgpr_spills"] > 0) <= 10


@pytest.mark.parametrize("parts,min_waves", [
    (("decode_stream_kernelILi4ELi2ELi1ELb0ELi0ELi2ELi0E",), 4),      # workload 2: 4-bit, K = 4096, two rows per wave
    (("decode_stream_kernelILi4ELi1ELi2ELb0ELi0ELi1ELi0E",), 4),      # workload 1: K = 1024
    (("decode_stream_kernelILi3ELi2ELi1ELb0ELi1ELi2ELi0E",), 4),      # workload 3: V2a 3-bit
    (("decode_stream_kernelILi3ELi2ELi1ELb0ELi2ELi2ELi0E",), 4),      # the same with a scale and a mid-point per group
    (("decode_stream_kernelILi3ELi2ELi1ELb0ELi0ELi4ELi0E",), 4),      # workload 4 gate_up
    (("decode_stream_kernelILi3ELi1ELi2ELb0ELi0ELi4ELi0E",), 4),      # workload 4 down
    (("decode_batch_kernelILi4ELi0ELi8ELi8ELb0ELb0E",), 1),           # workload 5: 8 waves, 8 groups each
    (("decode_tile_kernelILi4ELi16ELb0E",), 4),                       # 8192 x 28672: sixteen waves, one tile per CU
    (("decode_tile_kernelILi4ELi8ELb0E",), 4),                        # large 4-bit matrices: two workgroups per CU
    (("decode_wide_kernelILi4ELi4ELi0E",), 4),                        # 64 tokens in one pass: two workgroups per CU
    (("decode_wide_kernelILi4ELi2ELi0E",), 4),
    (("decode_wide_kernelILi3ELi4ELi0E",), 4),
    (("decode_wide_kernelILi3ELi4ELi1E",), 4),                        # V2a
    (("decode_wide_kernelILi4ELi4ELi1E",), 4),
    (("decode_wide_kernelILi4ELi1ELi2E",), 4),                        # V2a with a scale and a mid-point per group, 16 tokens
    (("decode_wide_kernelILi3ELi1ELi2E",), 4),
])
def test_the_workloads_kernels_keep_their_registers(parts, min_waves):
    k = find(resources(), *parts)
    assert k["vgpr_spills"] == 0 and k["scratch_bytes_per_lane"] == 0, k
    assert k["waves_per_simd"] >= min_waves, k


def test_kernels_that_address_lds_from_zero_have_no_static_lds():
    """The matrix-core kernels, the tile kernel and the V2a streaming kernels form lookup addresses that assume
    their tables at LDS offset 0 (one v_perm_b32 writes the whole address).  That holds because they declare
    dynamic LDS only; a static __shared__ array added to one of them would move the tables and the kernel would
    return without writing (its guard).  This pins the guarantee at build time."""
    res = resources()
    names = [k for k in res if any(p in k for p in ("decode_batch_kernel", "decode_tile_kernel", "decode_wide_kernel"))]
    # the streaming kernel's V2a instantiations: template argument 5 (MODE) is 1, or 2 with a scale and a mid-point per group
    names += [k for k in res if "decode_stream_kernelILi" in k and k.split("decode_stream_kernelI")[1].split("E")[4] in ("Li1", "Li2")]
    assert len(names) >= 100
    for k in names:
        assert res[k]["lds_bytes"] == 0, (k, res[k])
