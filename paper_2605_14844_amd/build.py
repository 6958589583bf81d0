"""Build libxfp.so (hipcc, gfx950 only) in-tree next to this file."""
from __future__ import annotations

import glob
import hashlib
import json
import os
import re
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libxfp.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-Rpass-analysis=kernel-resource-usage",      # registers, spills, LDS of every kernel -> kernel_resources.json
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


RESOURCES = os.path.join(HERE, "kernel_resources.json")


def _resources(text):
    """Per-kernel figures from the compiler's resource-usage remarks: {mangled name: {vgprs, spills, ...}}."""
    res = {}
    for blk in text.split("Function Name: ")[1:]:
        name = blk.split()[0]
        num = lambda key: int(m.group(1)) if (m := re.search(key + r": (\d+)", blk)) else -1
        res[name] = {"vgprs": num("VGPRs"), "agprs": num("AGPRs"), "sgprs": num("SGPRs"), "vgpr_spills": num("VGPRs Spill"),
                     "sgpr_spills": num("SGPRs Spill"), "scratch_bytes_per_lane": num(r"ScratchSize \[bytes/lane\]"),
                     "waves_per_simd": num(r"Occupancy \[waves/SIMD\]"), "lds_bytes": num(r"LDS Size \[bytes/block\]")}
    return res


def _run(cmd, verbose, remarks_to=None):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if remarks_to is not None and res.returncode == 0:
        with open(remarks_to, "w") as f:
            json.dump(_resources(res.stdout), f)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "-Rpass-analysis" not in l and not l.startswith(("remark:", "  ")) and "remark:" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and out.strip():
        print(out)


def _stamp(src: str) -> str:
    """Hash of everything an object depends on: flags, the source, every header."""
    h = hashlib.sha1(" ".join(HIPCC_FLAGS).encode())
    deps = [src] + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + sorted(glob.glob(os.path.join(HERE, "..", "include", "*.h")))
    for d in deps:
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compile every source to an object (in parallel), link, then replace the library atomically.
    incremental: reuse objects of unchanged sources from _build/ (a development convenience; the
    default compiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmpdir = tempfile.mkdtemp(prefix="xfp_build_")
    cache = os.path.join(HERE, "_build")
    try:
        objs = []
        jobs = []
        for src in sources():
            name = os.path.basename(src)[:-4]
            if incremental:
                os.makedirs(cache, exist_ok=True)
                obj = os.path.join(cache, f"{name}.{_stamp(src)}.o")
                if not os.path.exists(obj):
                    for old in glob.glob(os.path.join(cache, name + ".*.o*")):
                        os.remove(old)
                    jobs.append([hipcc, *HIPCC_FLAGS, "-c", "-o", obj, src])
            else:
                obj = os.path.join(tmpdir, name + ".o")
                jobs.append([hipcc, *HIPCC_FLAGS, "-c", "-o", obj, src])
            objs.append(obj)
        workers = max(1, min(len(jobs), os.cpu_count() or 1, 8))
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(lambda c: _run(c, verbose, remarks_to=c[c.index("-o") + 1] + ".json"), jobs))
        merged = {}
        for obj in objs:
            if os.path.exists(obj + ".json"):
                with open(obj + ".json") as f:
                    merged.update(json.load(f))
        with open(RESOURCES, "w") as f:
            json.dump(merged, f, indent=0, sort_keys=True)
        tmp = LIB + f".tmp{os.getpid()}"
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], verbose)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))
