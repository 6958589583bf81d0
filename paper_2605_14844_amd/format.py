"""The .xfp packed-weight file and the storage-size model.

The paper caches packed weights on disk after the first quantize-on-load
(section 4.5) but gives no file layout; this one is this library's own:

    bytes 0..7    magic  b"XFPMI355"
    bytes 8..11   uint32 version (1)
    bytes 12..15  uint32 header length H (JSON, UTF-8), header starts at byte 16
    then          sections, each starting at a multiple of 256 bytes, in the
                  order given by the header's "sections" list

The JSON header carries mode, bits, group, N, K, L, E and, per section, name,
dtype, shape and byte offset.  Section contents are exactly the arrays that
include/xfp.h describes, so a loaded file can be uploaded unchanged.
"""
from __future__ import annotations

import json
from types import SimpleNamespace

import numpy as np

MAGIC = b"XFPMI355"
VERSION = 1
ALIGN = 256
_SECTIONS = ("indices", "codebooks", "group_ids", "out_row_ptr", "out_col", "out_val", "group_scale", "group_mid")


def save_xfp(path: str, W) -> None:
    meta = dict(mode=int(W.mode), bits=int(W.bits), group=int(W.group), N=int(W.N), K=int(W.K),
                L=int(W.L), E=int(W.E), sections=[])
    arrays = []
    for name in _SECTIONS:
        a = getattr(W, name, None)
        if a is None:
            continue
        a = np.ascontiguousarray(a)
        arrays.append(a)
        meta["sections"].append(dict(name=name, dtype=a.dtype.str, shape=list(a.shape), offset=0))
    # offsets depend on the header length, which depends on the offsets' digits: fix point
    hdr_len = 0
    for _ in range(4):
        pos = 16 + hdr_len
        for sec, a in zip(meta["sections"], arrays):
            pos = (pos + ALIGN - 1) // ALIGN * ALIGN
            sec["offset"] = pos
            pos += a.nbytes
        hdr = json.dumps(meta).encode()
        if len(hdr) == hdr_len:
            break
        hdr_len = len(hdr)
    with open(path, "wb") as f:
        f.write(MAGIC)
        f.write(np.array([VERSION, len(hdr)], dtype="<u4").tobytes())
        f.write(hdr)
        for sec, a in zip(meta["sections"], arrays):
            f.write(b"\0" * (sec["offset"] - f.tell()))
            f.write(a.tobytes())


def load_xfp(path: str, mmap: bool = True):
    """Read a .xfp file; arrays are memory-mapped (read-only) unless mmap=False."""
    with open(path, "rb") as f:
        head = f.read(16)
        if head[:8] != MAGIC:
            raise ValueError("not an .xfp file")
        version, hdr_len = np.frombuffer(head[8:], dtype="<u4")
        if version != VERSION:
            raise ValueError(f"unsupported .xfp version {version}")
        meta = json.loads(f.read(int(hdr_len)).decode())
    out = SimpleNamespace(**{k: meta[k] for k in ("mode", "bits", "group", "N", "K", "L", "E")})
    for name in _SECTIONS:
        setattr(out, name, None)
    for sec in meta["sections"]:
        if sec["offset"] % ALIGN:
            raise ValueError("misaligned section")
        shape = tuple(sec["shape"])
        dt = np.dtype(sec["dtype"])
        if int(np.prod(shape)) == 0:
            a = np.zeros(shape, dtype=dt)
        elif mmap:
            a = np.memmap(path, dtype=dt, mode="r", offset=sec["offset"], shape=shape)
        else:
            a = np.fromfile(path, dtype=dt, count=int(np.prod(shape)), offset=sec["offset"]).reshape(shape)
        setattr(out, sec["name"], a)
    wpr = out.K * out.bits // 32
    if out.indices.shape != (out.E, out.N, wpr):
        raise ValueError("indices section does not match the header's shape")
    if out.out_row_ptr.shape != (out.E * out.N + 1,):
        raise ValueError("out_row_ptr section does not match the header's shape")
    return out


def bytes_per_weight(bits: int, outlier_fraction: float = 0.0, outlier_bytes: float = 6.0,
                     mode: int = 0, K: int = 0, group: int = 128, group_record_bits: float = 8.0) -> float:
    """Storage per weight: packed indices + codebook share + outliers.

    outlier_bytes = 18 reproduces the paper's COO triples (section 3.2); this
    library's CSR stores 6 bytes per outlier.  For V2a the per-group record is
    group_record_bits / group (the paper's id + scale + mid-point is 40 bits).
    """
    b = bits / 8.0 + outlier_fraction * outlier_bytes
    if mode == 0:
        if K:
            b += (1 << bits) * 2.0 / K
    else:
        b += group_record_bits / 8.0 / group
    return b
