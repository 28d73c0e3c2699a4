"""ctypes front end of the CPU oracle (oracle/ccoll_szx_ref.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the bench's
cpu_baseline leg.  The product package never imports this module, and this
module never imports the product package.

`build()` compiles the oracle with g++; `lib()` loads it (building on demand).
All functions take and return numpy arrays on the host.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ccoll_szx_ref.cpp")
_SO = os.path.join(_HERE, "libccoll_szx_ref.so")

OK, EINVAL, ENOSPC, ECORRUPT = 0, -1, -2, -3
BLOCK, CHUNK = 128, 5120

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle shared library next to its source."""
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(_SRC):
        return _SO
    cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-Wall",
           "-shared", "-fPIC", _SRC, "-o", _SO]
    subprocess.run(cmd, check=True)
    return _SO


def _declare(L: ctypes.CDLL) -> ctypes.CDLL:
    c_sz, c_vp, c_f = ctypes.c_size_t, ctypes.c_void_p, ctypes.c_float
    L.ccoll_ref_max_compressed_bytes.restype = c_sz
    L.ccoll_ref_max_compressed_bytes.argtypes = [c_sz]
    L.ccoll_ref_compress_stats.restype = ctypes.c_int
    L.ccoll_ref_compress_stats.argtypes = [c_vp, c_sz, c_f, c_vp, c_sz, ctypes.POINTER(c_sz), c_vp]
    L.ccoll_ref_compress.restype = ctypes.c_int
    L.ccoll_ref_compress.argtypes = [c_vp, c_sz, c_f, c_vp, c_sz, ctypes.POINTER(c_sz)]
    L.ccoll_ref_decompress.restype = ctypes.c_int
    L.ccoll_ref_decompress.argtypes = [c_vp, c_sz, c_vp, c_sz]
    L.ccoll_ref_decompress_range.restype = ctypes.c_int
    L.ccoll_ref_decompress_range.argtypes = [c_vp, c_sz, c_sz, c_sz, c_vp]
    L.ccoll_ref_reduce_step_op.restype = ctypes.c_int
    L.ccoll_ref_reduce_step_op.argtypes = [ctypes.c_int, c_vp, c_sz, c_vp, c_sz, c_f, c_vp, c_sz, ctypes.POINTER(c_sz)]
    L.ccoll_ref_reduce_step.restype = ctypes.c_int
    L.ccoll_ref_reduce_step.argtypes = [c_vp, c_sz, c_vp, c_sz, c_f, c_vp, c_sz, ctypes.POINTER(c_sz)]
    L.ccoll_ref_classify_block.restype = ctypes.c_int
    L.ccoll_ref_classify_block.argtypes = [c_vp, ctypes.c_int, c_f, ctypes.POINTER(ctypes.c_int),
                                           ctypes.POINTER(c_f), ctypes.POINTER(ctypes.c_int)]
    return L


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = _declare(ctypes.CDLL(_SO))
    return _lib


def build_variant(edits, out_dir: str) -> ctypes.CDLL:
    """Mutation testing of the pins: compiles a copy of the oracle source with the given (old, new) text
    replacements, each of which must match exactly once, and returns the loaded library."""
    text = open(_SRC).read()
    for old, new in edits:
        if text.count(old) != 1:
            raise ValueError(f"edit does not match exactly once: {old!r}")
        text = text.replace(old, new)
    tag = "%08x" % (hash(tuple(edits)) & 0xffffffff)
    src = os.path.join(out_dir, f"ccoll_szx_ref_{tag}.cpp")
    so = os.path.join(out_dir, f"libccoll_szx_ref_{tag}.so")
    with open(src, "w") as f:
        f.write(text)
    subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", src, "-o", so],
                   check=True)
    return _declare(ctypes.CDLL(so))


class use_library:
    """Context manager: the module's functions call library L inside the block (the pins run against a variant)."""

    def __init__(self, L: ctypes.CDLL):
        self.L = L

    def __enter__(self):
        global _lib
        lib()
        self.saved, _lib = _lib, self.L
        return self.L

    def __exit__(self, *exc):
        global _lib
        _lib = self.saved
        return False


class RefError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle returned {code}")
        self.code = code


def _f32(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32)


def _u8(b) -> np.ndarray:
    return np.ascontiguousarray(np.frombuffer(b, dtype=np.uint8) if isinstance(b, (bytes, bytearray)) else b,
                                dtype=np.uint8)


def max_compressed_bytes(n: int) -> int:
    return int(lib().ccoll_ref_max_compressed_bytes(n))


def compress(x, abs_eb: float, cap: int | None = None, with_counts: bool = False):
    """Returns the stream as a uint8 array (and [const, nonconst, raw] block counts)."""
    x = _f32(x).ravel()
    n = x.size
    if cap is None:
        cap = max_compressed_bytes(n)
    out = np.empty(max(cap, 1), dtype=np.uint8)
    nbytes = ctypes.c_size_t(0)
    counts = np.zeros(3, dtype=np.int64)
    rc = lib().ccoll_ref_compress_stats(x.ctypes.data, n, float(np.float32(abs_eb)), out.ctypes.data, cap,
                                        ctypes.byref(nbytes), counts.ctypes.data)
    if rc:
        raise RefError(rc)
    stream = out[: nbytes.value].copy()
    return (stream, counts) if with_counts else stream


def decompress(stream, n: int, in_bytes: int | None = None) -> np.ndarray:
    s = _u8(stream)
    out = np.empty(max(n, 1), dtype=np.float32)
    rc = lib().ccoll_ref_decompress(s.ctypes.data, s.size if in_bytes is None else in_bytes, out.ctypes.data, n)
    if rc:
        raise RefError(rc)
    return out[:n]


def decompress_range(stream, first: int, count: int) -> np.ndarray:
    s = _u8(stream)
    out = np.empty(max(count, 1), dtype=np.float32)
    rc = lib().ccoll_ref_decompress_range(s.ctypes.data, s.size, first, count, out.ctypes.data)
    if rc:
        raise RefError(rc)
    return out[:count]


OPS = {"sum": 0, "max": 1, "min": 2}


def reduce_step(local, cin, abs_eb: float, cap: int | None = None, op: str = "sum") -> np.ndarray:
    x = _f32(local).ravel()
    s = _u8(cin)
    n = x.size
    if cap is None:
        cap = max_compressed_bytes(n)
    out = np.empty(max(cap, 1), dtype=np.uint8)
    nbytes = ctypes.c_size_t(0)
    rc = lib().ccoll_ref_reduce_step_op(OPS[op], x.ctypes.data, n, s.ctypes.data, s.size, float(np.float32(abs_eb)),
                                        out.ctypes.data, cap, ctypes.byref(nbytes))
    if rc:
        raise RefError(rc)
    return out[: nbytes.value].copy()


def classify_block(x, abs_eb: float):
    """(type, mu, reqlen) of one block; type 0 CONST, 1 NONCONST, 2 RAW."""
    x = _f32(x).ravel()
    t, mu, rq = ctypes.c_int(0), ctypes.c_float(0), ctypes.c_int(0)
    rc = lib().ccoll_ref_classify_block(x.ctypes.data, x.size, float(np.float32(abs_eb)), ctypes.byref(t),
                                        ctypes.byref(mu), ctypes.byref(rq))
    if rc:
        raise RefError(rc)
    return t.value, np.float32(mu.value), rq.value


if __name__ == "__main__":
    print(build(force=True))
