"""Writer (and a numpy reader) of the serialized index file that the library and the CPU oracle both load.

Layout (little-endian; every array starts at a multiple of 64 bytes from the start of the file):

    offset  0  char[8]  magic "LRNIDX01"
            8  int32    metric (0 inner product, 1 squared Euclidean, 2 cosine)
           12  int32    d        16  int32  dp (d')     20  int32  r      24  int32  L
           28  int32    flags    bit 0: a projection matrix follows; bit 1: ids follow
           32  int64    n
           40  zero padding up to 64
    then, in this order: cluster_offsets int64[L+1]; ids int64[n] (if flagged); centroids float[L][dp];
    P float[d][dp] (if flagged); A int8[L][r][dp]; B int8[n][r]; scale_A float[L]; scale_B float[L];
    corpus float[n][d].

The arrays have exactly the layouts of the load call of the C interface.
"""
from __future__ import annotations

import struct

import numpy as np

MAGIC = b"LRNIDX01"
_ALIGN = 64


def _sections(h):
    n, d, dp, r, L = h["n"], h["d"], h["dp"], h["r"], h["L"]
    out = [("cluster_offsets", np.int64, (L + 1,))]
    if h["has_ids"]:
        out.append(("ids", np.int64, (n,)))
    out.append(("centroids", np.float32, (L, dp)))
    if h["has_P"]:
        out.append(("P", np.float32, (d, dp)))
    out += [("A", np.int8, (L, r, dp)), ("B", np.int8, (n, r)), ("scale_A", np.float32, (L,)),
            ("scale_B", np.float32, (L,)), ("corpus", np.float32, (n, d))]
    return out


def _host(a, dtype):
    if a is None:
        return None
    if hasattr(a, "detach"):
        a = a.detach().cpu().numpy()
    return np.ascontiguousarray(a, dtype=dtype)


def save_index(path, ix) -> None:
    """Write `ix` (a synth.IndexArrays or a dict with the same field names) to `path`."""
    get = (lambda k: ix.get(k)) if isinstance(ix, dict) else (lambda k: getattr(ix, k))
    h = dict(metric=int(get("metric")), n=int(get("n")), d=int(get("d")), dp=int(get("dp")), r=int(get("r")),
             L=int(get("L")), has_P=get("P") is not None, has_ids=get("ids") is not None)
    with open(path, "wb") as f:
        head = MAGIC + struct.pack("<6i", h["metric"], h["d"], h["dp"], h["r"], h["L"],
                                   (1 if h["has_P"] else 0) | (2 if h["has_ids"] else 0)) + struct.pack("<q", h["n"])
        f.write(head + b"\0" * (_ALIGN - len(head)))
        for name, dtype, shape in _sections(h):
            a = _host(get(name), dtype)
            if a.shape != shape:
                raise ValueError(f"{name}: shape {a.shape}, expected {shape}")
            pos = f.tell()
            f.write(b"\0" * ((-pos) % _ALIGN))
            f.write(a.astype(np.dtype(dtype).newbyteorder("<"), copy=False).tobytes())


def read_header(path) -> dict:
    """The header fields of a file written by save_index."""
    with open(path, "rb") as f:
        head = f.read(_ALIGN)
    if len(head) < _ALIGN or head[:8] != MAGIC:
        raise ValueError("not a LRNIDX01 file")
    metric, d, dp, r, L, flags = struct.unpack("<6i", head[8:32])
    (n,) = struct.unpack("<q", head[32:40])
    return dict(metric=metric, n=n, d=d, dp=dp, r=r, L=L, has_P=bool(flags & 1), has_ids=bool(flags & 2))


def read_index(path) -> dict:
    """Read a file written by save_index into a dict of numpy arrays (memory-mapped, read-only)."""
    h = read_header(path)
    metric, n, d, dp, r, L = (h[k] for k in ("metric", "n", "d", "dp", "r", "L"))
    out = dict(metric=metric, n=n, d=d, dp=dp, r=r, L=L, P=None, ids=None)
    pos = _ALIGN
    for name, dtype, shape in _sections(h):
        pos += (-pos) % _ALIGN
        out[name] = np.memmap(path, dtype=np.dtype(dtype).newbyteorder("<"), mode="r", offset=pos, shape=shape)
        pos += int(np.prod(shape)) * np.dtype(dtype).itemsize
    return out
