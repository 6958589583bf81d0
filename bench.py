#!/usr/bin/env python3
"""Benchmark of the XFP fused decode path on one MI355X.

A step is one pass of the whole hot path over one batch: one xfp_gemv call
(workloads 1, 2, 3, 5) or one gate_up + one down xfp_gemv_moe call (workload
4).  More configurations measure what was added beyond the five: 6 (the
expert layer of workload 4 with both epilogues fused), 7 (long rows), 8-10 (the
batched kernel's other forms), 11 (2 bits).  Weights are already resident in
HBM; successive steps walk a ring of distinct device copies whose total size
exceeds the last-level cache, and 768 MB are streamed through the chip right
before the timed steps, so the weights of a step are never cache-resident,
whatever --steps is.  Up to 512 timed steps are eager launches that the GPU
finds already queued (they are submitted while the flush kernels run), bracketed
by two events on the launch stream; longer runs are recorded into one HIP graph
and replayed once between two events (a graph launch has a fixed cost of about
12 us on this stack, which a short run would charge to its few steps; the
replay's figure is reported beside the other).  The eager launch rate from
Python is reported too.

Prints ONE JSON line.  value = algorithmic bytes per step / time per step of
the headline workload (2); the default run adds the same figures for workloads
1, 3, 4, 5 and the 2-bit matrix under "configs".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
RING_BYTES = 1 << 30


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=2000)
    p.add_argument("--warmup", type=int, default=200)
    p.add_argument("--config", type=int, default=2,
                   help="workload 1..5 (default 2, the headline); beyond the five: 6 = workload 4 as a whole expert "
                        "layer with both epilogues fused, 7 = a long-row matrix (8192x28672, 4-bit, M=1) through the tile kernel, "
                        "8 = the same matrix with 16 tokens, 9 = workload 5's shape at 3 bits, 10 = the same as V2a, "
                        "11 = workload 2's shape at 2 bits, 12 = workload 5's matrix with 64 tokens (wide matrix-core kernel), 13 = configuration 10's matrix with 64 tokens, 14 = workload 3's shape with a scale and a mid-point per group, 15 = configuration 10 with them")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--single", action="store_true", help="time only --config (the default run of workload 2 also "
                   "times workloads 1, 3, 4, 5 and a 2-bit matrix and reports them under \"configs\")")
    p.add_argument("--no-graph", action="store_true", help="time eager launches instead of a graph")
    p.add_argument("--no-plain-read", action="store_true", help="skip the read-only ceiling measurement")
    p.add_argument("--ring-bytes", type=int, default=RING_BYTES)
    p.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                   help="instead of the benchmark, run xfp_probe_copy over MIB mebibytes 20 times "
                        "(known traffic, used to scale the profiler's FETCH_SIZE / WRITE_SIZE)")
    return p.parse_args()


def build_workload(cfg: int, ring_bytes: int):
    """Returns dict(name, step(i), bytes, ring, oracle(), launches_per_step, kernel_bytes)."""
    import numpy as np
    import torch

    import paper_2605_14844_amd as xfp
    import xfp_inputs as xi

    def dev_x(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.float16)

    def clone_weights(dW):
        t = {k: (None if v is None else v.clone()) for k, v in dW.tensors.items()}
        d = dW.desc
        return xfp.binding.make_descriptor(d.mode, d.bits, d.N, d.K, d.L, d.E, t["indices"],
                                           t["codebooks"], t["group_ids"], t["out_row_ptr"],
                                           t["out_col"], t["out_val"], group_scale=t.get("group_scale"),
                                           group_mid=t.get("group_mid"))

    if cfg in (1, 2, 3, 5):
        M = 16 if cfg == 5 else 1
        W = xi.config_weights(cfg)
        xb = xi.config_x(cfg, M, W.K)
        nbytes = W.algorithmic_bytes(M=M)
        R = max(1, min(512, -(-ring_bytes // nbytes)))
        ring = [xfp.upload(W)]
        for _ in range(R - 1):
            ring.append(clone_weights(ring[0]))
        xd = dev_x(xb)
        y = torch.empty((M, W.N), dtype=torch.float16, device="cuda")

        def step(i):
            xfp.xfp_gemv(ring[i % R], xd, y=y)

        def oracle_once(threads=None):
            import oracle
            return oracle.gemv_weights(W, xb, threads)

        return dict(name=xi.CONFIG_NAMES[cfg], step=step, bytes=nbytes, ring=R, oracle=oracle_once,
                    launches=1 if M == 1 else 2,      # M > 1: x relayout kernel, then the decode kernel
                    kernel_bytes=nbytes, launch_bytes=[nbytes], keep=(ring, xd, y), M=M, N=W.N, K=W.K,
                    bits=W.bits, mode=W.mode)

    if cfg == 4:
        T = 8
        gu, dn = xi.config_weights(4)
        dgu, ddn = xfp.upload(gu), xfp.upload(dn)
        draws = 64
        ids_host = [xi.config_expert_ids(4, T, gu.E, draw=d) for d in range(draws)]
        ids_dev = [torch.from_numpy(a).cuda() for a in ids_host]
        x1b = xi.config_x(4, 1, gu.K)
        x2b = xi.activations(np.random.default_rng(xi.BASE_SEED + 404), T, dn.K)
        x1, x2 = dev_x(x1b)[0], dev_x(x2b)
        y1 = torch.empty((T, gu.N), dtype=torch.float16, device="cuda")
        y2 = torch.empty((T, dn.N), dtype=torch.float16, device="cuda")
        b1 = gu.algorithmic_bytes(experts=T, shared_x=True)
        b2 = dn.algorithmic_bytes(experts=T, shared_x=False)

        def step(i):
            ids = ids_dev[i % draws]
            xfp.xfp_gemv_moe(dgu, ids, x1, y=y1)
            xfp.xfp_gemv_moe(ddn, ids, x2, y=y2)

        def oracle_once(threads=None):
            import oracle
            a = oracle.gemv_moe(gu, ids_host[0], x1b, True, threads)
            b = oracle.gemv_moe(dn, ids_host[0], x2b, False, threads)
            return a, b

        return dict(name=xi.CONFIG_NAMES[4], step=step, bytes=b1 + b2, ring=draws, oracle=oracle_once,
                    launches=2, kernel_bytes=b1, launch_bytes=[b1, b2], keep=(dgu, ddn, ids_dev, x1, x2, y1, y2), M=1,
                    N=gu.N, K=gu.K, bits=3, mode=0)
    if cfg == 6:
        # workload 4 as an expert layer: gate/up with SiLU(gate)*up in the store, then the down projection
        # with the router's weighted sum; the intermediate h feeds the second call (two launches per step)
        T = 8
        gu, dn = xi.config_weights(4)
        dgu, ddn = xfp.upload(gu), xfp.upload(dn)
        draws = 64
        ids_host = [xi.config_expert_ids(4, T, gu.E, draw=d) for d in range(draws)]
        ids_dev = [torch.from_numpy(a).cuda() for a in ids_host]
        x1b = xi.config_x(4, 1, gu.K)
        x1 = dev_x(x1b)[0]
        w_host = np.random.default_rng(xi.BASE_SEED + 406).random(T).astype(np.float32)
        w_host /= w_host.sum()
        w_dev = torch.from_numpy(w_host).cuda()
        h = torch.empty((T, gu.N // 2), dtype=torch.float16, device="cuda")
        y = torch.empty((dn.N,), dtype=torch.float16, device="cuda")
        assert gu.N // 2 == dn.K
        b1 = gu.algorithmic_bytes(experts=T, shared_x=True) - T * gu.N * 2 + T * (gu.N // 2) * 2   # h instead of y
        b2 = dn.algorithmic_bytes(experts=T, shared_x=False) - T * dn.N * 2 + dn.N * 2 + T * 4     # one y, T weights

        def step(i):
            ids = ids_dev[i % draws]
            xfp.xfp_gemv_moe_silu_mul(dgu, ids, x1, h=h)
            xfp.xfp_gemv_moe_combine(ddn, ids, h, w_dev, y=y)

        def oracle_once(threads=None):
            import oracle
            hh = oracle.silu_mul(oracle.gemv_moe(gu, ids_host[0], x1b, True, threads))
            hb = hh.astype(np.float16).view(np.uint16)
            return oracle.moe_combine(oracle.gemv_moe(dn, ids_host[0], hb, False, threads), w_host)

        return dict(name="expert layer of workload 4: gate_up with SiLU(gate)*up, down with the router's combine",
                    step=step, bytes=b1 + b2, ring=draws, oracle=oracle_once, launches=2, kernel_bytes=b1,
                    launch_bytes=[b1, b2], keep=(dgu, ddn, ids_dev, x1, h, y, w_dev), M=1, N=gu.N, K=gu.K, bits=3,
                    mode=0)

    if cfg == 7:
        W = xi.random_weights(xi.MODE_V2, 4, 8192, 28672, density=0.003, seed=xi.BASE_SEED + 7)
        xb = xi.activations(np.random.default_rng(xi.BASE_SEED + 407), 1, W.K)
        nbytes = W.algorithmic_bytes(M=1)
        R = max(1, min(512, -(-ring_bytes // nbytes)))
        ring = [xfp.upload(W)]
        for _ in range(R - 1):
            ring.append(clone_weights(ring[0]))
        xd = dev_x(xb)
        y = torch.empty((1, W.N), dtype=torch.float16, device="cuda")

        def step(i):
            xfp.xfp_gemv(ring[i % R], xd, y=y)

        def oracle_once(threads=None):
            import oracle
            return oracle.gemv_weights(W, xb, threads)

        return dict(name="V2 8192x28672 b4 M=1 (rows longer than 16384: the tile kernel, one launch)", step=step,
                    bytes=nbytes, ring=R, oracle=oracle_once, launches=1, kernel_bytes=nbytes,
                    launch_bytes=[nbytes], keep=(ring, xd, y), M=1, N=W.N, K=W.K, bits=4, mode=0)
    if cfg in (11, 14):
        if cfg == 11:
            W = xi.random_weights(xi.MODE_V2, 2, 8192, 4096, density=0.003, seed=xi.BASE_SEED + 11)
        else:
            W = xi.random_weights(xi.MODE_V2A, 3, 4096, 4096, L=32, density=0.001, seed=xi.BASE_SEED + 14, affine=True)
        xb = xi.activations(np.random.default_rng(xi.BASE_SEED + 400 + cfg), 1, W.K)
        nbytes = W.algorithmic_bytes(M=1)
        R = max(1, min(512, -(-ring_bytes // nbytes)))
        ring = [xfp.upload(W)]
        for _ in range(R - 1):
            ring.append(clone_weights(ring[0]))
        xd = dev_x(xb)
        y = torch.empty((1, W.N), dtype=torch.float16, device="cuda")

        def step(i):
            xfp.xfp_gemv(ring[i % R], xd, y=y)

        def oracle_once(threads=None):
            import oracle
            return oracle.gemv_weights(W, xb, threads)

        name = ("V2 8192x4096 b2 M=1 (workload 2's shape at 2 bits)" if cfg == 11 else
                "V2a 4096x4096 b3 L=32 M=1 with a scale and a mid-point per group (workload 3's shape in the paper's 40-bit group record)")
        return dict(name=name, step=step, bytes=nbytes, ring=R,
                    oracle=oracle_once, launches=1, kernel_bytes=nbytes, launch_bytes=[nbytes], keep=(ring, xd, y),
                    M=1, N=W.N, K=W.K, bits=W.bits, mode=W.mode)
    if cfg in (8, 9, 10, 15):
        if cfg == 8:
            W = xi.random_weights(xi.MODE_V2, 4, 8192, 28672, density=0.003, seed=xi.BASE_SEED + 7)
        elif cfg == 9:
            W = xi.random_weights(xi.MODE_V2, 3, 28672, 8192, density=0.003, seed=xi.BASE_SEED + 9)
        else:
            W = xi.random_weights(xi.MODE_V2A, 3, 28672, 8192, L=32, density=0.003, seed=xi.BASE_SEED + 10, affine=cfg == 15)
        xb = xi.activations(np.random.default_rng(xi.BASE_SEED + 400 + cfg), 16, W.K)
        nbytes = W.algorithmic_bytes(M=16)
        R = max(1, min(512, -(-ring_bytes // nbytes)))
        ring = [xfp.upload(W)]
        for _ in range(R - 1):
            ring.append(clone_weights(ring[0]))
        xd = dev_x(xb)
        y = torch.empty((16, W.N), dtype=torch.float16, device="cuda")

        def step(i):
            xfp.xfp_gemv(ring[i % R], xd, y=y)

        def oracle_once(threads=None):
            import oracle
            return oracle.gemv_weights(W, xb, threads)

        name = {8: "V2 8192x28672 b4 M=16 (rows the 16-token kernel would slice: the wide matrix-core kernel, two launches)",
                9: "V2 28672x8192 b3 M=16 (workload 5's shape at 3 bits, two launches)",
                10: "V2a 28672x8192 b3 L=32 M=16 (workload 5's shape in workload 3's format, two launches)",
                15: "V2a 28672x8192 b3 L=32 M=16 with a scale and a mid-point per group (wide matrix-core kernel in its mode for flagged tensors, two launches)"}[cfg]
        return dict(name=name, step=step, bytes=nbytes, ring=R, oracle=oracle_once, launches=2,
                    kernel_bytes=nbytes, launch_bytes=[nbytes], keep=(ring, xd, y), M=16, N=W.N, K=W.K, bits=W.bits,
                    mode=W.mode)
    if cfg in (12, 13):
        # 64 tokens in one pass of the wide matrix-core kernel: workload 5's matrix (12), configuration 10's (13)
        if cfg == 12:
            W = xi.config_weights(5)
            xb = xi.config_x(5, 64, W.K)
            name = "V2 28672x8192 b4 M=64 (workload 5's matrix, 64 tokens in one pass: wide matrix-core kernel, two launches)"
        else:
            W = xi.random_weights(xi.MODE_V2A, 3, 28672, 8192, L=32, density=0.003, seed=xi.BASE_SEED + 10)
            xb = xi.activations(np.random.default_rng(xi.BASE_SEED + 413), 64, W.K)
            name = "V2a 28672x8192 b3 L=32 M=64 (configuration 10's matrix, 64 tokens in one pass: wide matrix-core kernel, two launches)"
        nbytes = W.algorithmic_bytes(M=64)
        R = max(1, min(512, -(-ring_bytes // nbytes)))
        ring = [xfp.upload(W)]
        for _ in range(R - 1):
            ring.append(clone_weights(ring[0]))
        xd = dev_x(xb)
        y = torch.empty((64, W.N), dtype=torch.float16, device="cuda")

        def step(i):
            xfp.xfp_gemv(ring[i % R], xd, y=y)

        def oracle_once(threads=None):
            import oracle
            return oracle.gemv_weights(W, xb, threads)

        return dict(name=name, step=step, bytes=nbytes, ring=R, oracle=oracle_once, launches=2, kernel_bytes=nbytes,
                    launch_bytes=[nbytes], keep=(ring, xd, y), M=64, N=W.N, K=W.K, bits=W.bits, mode=W.mode)
    raise SystemExit(f"no workload {cfg}")


def read_traffic(cfg: int):
    """HBM bytes per launch from an OFFLINE rocprofv3 --pmc run (see profiles/; not measured in this run),
    and where the figure comes from; (None, None) when no such file exists."""
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_workload{cfg}.txt")
    try:
        val, stamp = None, ""
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                val = float(line.split(":")[1].split()[0])
            if line.startswith("kernels_as_of:"):
                stamp = ", kernels as of " + line.split(":", 1)[1].strip()
        if val is not None:
            return val, f"offline: profiles/{os.path.basename(path)} (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE{stamp})"
    except OSError:
        pass
    return None, None


class CacheFlush:
    """Streams a buffer three times the size of the 256 MB last-level cache through the chip (read-only kernel),
    so that whatever the previous replay left in L2 / Infinity Cache is gone before a timed replay starts."""

    def __init__(self, nbytes=768 << 20):
        import torch
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.buf.random_(0, 256)
        self.sink = torch.zeros(4096, dtype=torch.int32, device="cuda")

    def launch(self):
        import paper_2605_14844_amd as xfp
        xfp.xfp_probe_read(self.buf, self.sink)

    def __call__(self):
        import torch
        self.launch()
        torch.cuda.synchronize()

    def spin_up(self, seconds=0.4):
        """Keeps the chip busy for a while: a GPU that has idled (set-up runs on the host) starts at low clocks and
        takes milliseconds of load to reach the ones it serves at; a run of a few dozen steps would otherwise be
        timed on the ramp."""
        import torch
        t = time.perf_counter()
        while time.perf_counter() - t < seconds:
            for _ in range(16):
                self.launch()
            torch.cuda.synchronize()


def timed_graph(step, K, first, flush):
    """Records steps first .. first + K - 1 into one HIP graph, replays it once untimed (the first replay
    uploads the graph), flushes the caches, then times ONE replay (exactly K steps) between two events on
    the launch stream.  Returns (ms per step by the events, ms per step by the host clock)."""
    import torch
    stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for i in range(K):
                step(first + i)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    flush()
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    g0.record(stream)
    graph.replay()
    g1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - w0) * 1e3 / K
    return g0.elapsed_time(g1) / K, wall_ms


QUEUED_MAX_STEPS = 512
def queued_repeats(K):
    """How often the K steps are timed (each time behind its own flush; the median is reported): a timing of 20
    steps lasts 0.1 ms and scatters by +-4 %, so short runs are repeated until about 1000 steps have been timed."""
    return max(3, min(51, 1000 // K) | 1)


def timed_queued(step, K, first, flush):
    """Times K eager launches that the GPU finds already queued: the cache-flush kernel is launched n times without a
    synchronize, the K steps are submitted while it runs, and two events on the launch stream bracket exactly the K
    steps.  The GPU then runs them back to back from the queue, cold caches, with neither the host's launch
    latency nor the fixed cost of a graph launch (about 12 us on this stack, i.e. 0.6 us per step of a 20-step
    replay) inside the events.  Valid only if the host had submitted everything before the GPU reached the first
    step: checked through the time the host still waits after its last launch; returns None if that cannot be
    had (the caller then times a graph replay instead).  Returns the ms per step of queued_repeats(K) such timings
    of the same K steps, in the order taken (the first one also pays what only a first touch costs)."""
    import torch
    stream = torch.cuda.current_stream()
    torch.cuda.synchronize()
    t = time.perf_counter()
    for i in range(8):
        step(first + i)
    host_us = (time.perf_counter() - t) * 1e6 / 8            # what the host needs to submit one step
    torch.cuda.synchronize()
    flush_us = 1e30                                          # the shortest of three: a first launch can take ten times as long
    for _ in range(3):
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        f0.record(stream)
        flush.launch()
        f1.record(stream)
        torch.cuda.synchronize()
        flush_us = min(flush_us, f0.elapsed_time(f1) * 1e3)
    n = int(1.5 * K * host_us / flush_us) + 3
    good = []
    repeats = queued_repeats(K)
    for _ in range(repeats + 2):
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        for _j in range(n):
            flush.launch()
        g0.record(stream)
        for i in range(K):
            step(first + i)
        g1.record(stream)
        t = time.perf_counter()
        torch.cuda.synchronize()
        waited_us = (time.perf_counter() - t) * 1e6
        ms = g0.elapsed_time(g1) / K
        if waited_us >= 1.2 * K * ms * 1e3 + 50.0:             # the whole timed region ran after the last launch
            good.append(ms)
            if len(good) == repeats:
                return good
        else:
            n *= 2
    return None


def timed_steps(step, K, first, flush):
    """(ms per step, ms per step by the host clock or None, how it was timed)."""
    if K <= QUEUED_MAX_STEPS:
        runs = timed_queued(step, K, first, flush)
        if runs is not None:
            srt = sorted(runs)
            how = ("eager launches already queued behind the cache-flush kernels, events on the launch stream; median of "
                   f"{len(runs)} timings of the same {K} steps (first {runs[0] * 1e3:.3f}, min {srt[0] * 1e3:.3f}, "
                   f"quartiles {srt[len(srt) // 4] * 1e3:.3f} / {srt[len(srt) // 2] * 1e3:.3f} / {srt[3 * len(srt) // 4] * 1e3:.3f}, "
                   f"max {srt[-1] * 1e3:.3f} us per step)")
            return srt[len(srt) // 2], None, how
    ms, wall = timed_graph(step, K, first, flush)
    return ms, wall, "hip graph replay"


def time_plain_read(launch_bytes, K, ring_bytes, flush):
    """us per step of xfp_probe_read over the same byte counts, one launch per decode launch, walking a
    buffer of ring_bytes so that no cache holds the data; same graph replay, flush and events as the decode."""
    import torch

    import paper_2605_14844_amd as xfp
    buf = torch.empty(ring_bytes + max(launch_bytes) + 4096, dtype=torch.uint8, device="cuda")
    buf.random_(0, 256)
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    state = {"off": 0}

    def step(_i):
        for nb in launch_bytes:
            nb16 = nb // 16 * 16
            if state["off"] + nb16 > ring_bytes:
                state["off"] = 0
            xfp.xfp_probe_read(buf[state["off"]:], sink, nbytes=nb16)
            state["off"] += (nb16 + 4095) // 4096 * 4096

    for i in range(20):
        step(i)
    return timed_steps(step, K, 0, flush)[0] * 1e3


def measure(cfg, args, flush, want_eager=True):
    """Builds workload cfg, runs warm-up, times K steps; returns (workload, dict of figures)."""
    import torch
    t0 = time.time()
    wl = build_workload(cfg, args.ring_bytes)
    setup_s = time.time() - t0
    step, K, Wm = wl["step"], args.steps, args.warmup
    stream = torch.cuda.current_stream()
    flush.spin_up()
    for i in range(Wm):
        step(i)
    torch.cuda.synchronize()
    eager_ms = None
    if want_eager or args.no_graph:
        # eager launch rate (reported, not the headline): Python + ctypes + hipLaunchKernel per call
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(K):
            step(Wm + i)
        e1.record(stream)
        torch.cuda.synchronize()
        eager_ms = e0.elapsed_time(e1) / K
    graph_ms = None
    if args.no_graph:
        ms_per_step, wall_ms, how = eager_ms, eager_ms, "eager"
    else:
        ms_per_step, wall_ms, how = timed_steps(step, K, Wm, flush)
        if how != "hip graph replay" and want_eager:
            graph_ms = timed_graph(step, K, Wm, flush)[0]     # reported beside it
    res = {"ms_per_step": ms_per_step, "wall_ms": wall_ms, "eager_ms": eager_ms, "setup_s": setup_s, "how": how,
           "graph_ms": graph_ms}
    if not args.no_graph and not args.no_plain_read:
        res["plain_read_us"] = time_plain_read(wl["launch_bytes"], K, args.ring_bytes, flush)
    return wl, res


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build covers the single-GPU decode kernel only; run with --gpus 1 "
              "(across GPUs the matrices would be sharded by output rows; no collective is involved).", file=sys.stderr)
        raise SystemExit(2)
    import torch

    import paper_2605_14844_amd as xfp
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    xfp.load_library()
    xfp.xfp_init()

    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.full((n,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(20):
            xfp.xfp_probe_copy(src, dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "launches": 20, "kernel": "probe_copy_kernel"}))
        return

    flush = CacheFlush()
    wl, res = measure(args.config, args, flush)
    K, Wm = args.steps, args.warmup
    ms_per_step = res["ms_per_step"]
    gbs = wl["bytes"] / (ms_per_step * 1e-3) / 1e9
    launch_ms = ms_per_step * wl["kernel_bytes"] / wl["bytes"] if wl["launches"] > 1 else ms_per_step
    achieved = wl["kernel_bytes"] / (launch_ms * 1e-3) / 1e9
    traffic, traffic_src = read_traffic(args.config)

    out = {
        "metric": "achieved HBM GB/s of the fused XFP decode GEMV (algorithmic bytes / time per call)",
        "value": round(gbs, 2), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 inputs, f32 accumulate", "data": "synthetic",
        "config": {"workload": wl["name"], "M": wl["M"], "N": wl["N"], "K": wl["K"], "bits": wl["bits"],
                   "mode": "V2a" if wl["mode"] else "V2", "y_dtype": "f16",
                   "algorithmic_bytes_per_step": wl["bytes"], "ring_copies": wl["ring"],
                   "launches_per_step": wl["launches"], "timed_with": res["how"],
                   "caches": "768 MB streamed through the chip right before the timed steps"},
        "us_per_call": round(ms_per_step * 1e3, 3),
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "eager_us_per_step": round(res["eager_ms"] * 1e3, 3),
        "wall_us_per_step": None if res["wall_ms"] is None else round(res["wall_ms"] * 1e3, 3),
        "graph_replay_us_per_step": None if res["graph_ms"] is None else round(res["graph_ms"] * 1e3, 3),
        "setup_s": round(res["setup_s"], 1),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_source": traffic_src},
    }
    if "plain_read_us" in res:
        pr_us = res["plain_read_us"]
        out["plain_read"] = {"us_per_step": round(pr_us, 3),
                             "GB/s": round(sum(b // 16 * 16 for b in wl["launch_bytes"]) / pr_us / 1e3, 2),
                             "decode_vs_plain_read": round(pr_us / (ms_per_step * 1e3), 4),
                             "kernel": "probe_read_kernel, one launch per decode launch, same bytes"}

    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.max_threads()
        wl["oracle"](threads)                # page in, build
        n, t1 = 0, time.perf_counter()
        while True:
            wl["oracle"](threads)
            n += 1
            dt = time.perf_counter() - t1
            if dt > 10.0 or n >= 5000:
                break
        out["cpu_baseline"] = {"value": round(wl["bytes"] * n / dt / 1e9, 4), "unit": "GB/s",
                               "cores": threads, "kind": "oracle",
                               "sample": f"{n} full calls of the same workload, {dt:.1f} s, "
                                         f"{dt / n * 1e3:.1f} ms per call"}

    if args.config == 2 and not args.single:
        # the other workloads of the target, same protocol, in the same line (the headline stays workload 2)
        table = {"C2": row_of(wl, res)}
        del wl
        for cfg in (1, 3, 4, 5, 11):
            torch.cuda.empty_cache()
            w2, r2 = measure(cfg, args, flush, want_eager=False)
            table[f"C{cfg}" if cfg <= 5 else "b2"] = row_of(w2, r2)
            del w2
        out["configs"] = table
    print(json.dumps(out))


def row_of(wl, res):
    us = res["ms_per_step"] * 1e3
    row = {"workload": wl["name"], "us_per_step": round(us, 3), "GB/s": round(wl["bytes"] / us / 1e3, 1),
           "frac": round(wl["bytes"] / us / 1e3 / HBM_PEAK_GBS, 4), "launches": wl["launches"],
           "algorithmic_bytes": wl["bytes"]}
    if "plain_read_us" in res:
        row["plain_read_us"] = round(res["plain_read_us"], 3)
    row["timed_with"] = res["how"].split(",")[0]
    return row


if __name__ == "__main__":
    main()
