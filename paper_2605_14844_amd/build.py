"""Build libxfp.so (hipcc, gfx950 only) in-tree next to this file."""
from __future__ import annotations

import glob
import hashlib
import os
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
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
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
                    for old in glob.glob(os.path.join(cache, name + ".*.o")):
                        os.remove(old)
                    jobs.append([hipcc, *HIPCC_FLAGS, "-c", "-o", obj, src])
            else:
                obj = os.path.join(tmpdir, name + ".o")
                jobs.append([hipcc, *HIPCC_FLAGS, "-c", "-o", obj, src])
            objs.append(obj)
        workers = max(1, min(len(jobs), os.cpu_count() or 1, 8))
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(lambda c: _run(c, verbose), jobs))
        tmp = LIB + f".tmp{os.getpid()}"
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], verbose)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))
