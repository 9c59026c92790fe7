"""ctypes wrapper around oracle/typemap_oracle.c.  TEST INFRASTRUCTURE ONLY.

Same role and same rules as oracle/typemap.py (see its header): the plain
type-map interpreter, here compiled so that the full-size workloads finish in
seconds and so the benchmark can time a CPU baseline.  Nothing in the product
path may import this module.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "typemap_oracle.c")
# TP_SANITIZE=address / thread: an instrumented build under a name of its own (for the CPU tests only;
# the loading process needs the sanitizer's runtime preloaded)
_SANITIZE = os.environ.get("TP_SANITIZE", "")
_SANITIZE_FLAGS = {"": [], "address": ["-fsanitize=address,undefined", "-fno-omit-frame-pointer"],
                   "thread": ["-fsanitize=thread", "-fno-omit-frame-pointer"]}[_SANITIZE]
_LIB = os.path.join(_HERE, f"libtypemap_oracle{'.' + _SANITIZE if _SANITIZE else ''}.so")

_NAMED_SIZE = {
    "BYTE": 1, "CHAR": 1, "INT8": 1, "UINT8": 1, "INT16": 2, "UINT16": 2,
    "INT32": 4, "UINT32": 4, "INT64": 8, "UINT64": 8, "FLOAT": 4, "DOUBLE": 8,
}
_KIND = {"named": 0, "contiguous": 1, "vector": 2, "hvector": 3, "subarray": 4}

_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (a checker, not part of the product)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-g", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", "-pthread", *_SANITIZE_FLAGS, _SRC,
             "-o", _LIB]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        i64, p64, pu8 = ctypes.c_int64, ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p
        lib.tmo_measure.argtypes = [p64, i64, p64, p64, p64]
        lib.tmo_measure.restype = ctypes.c_int
        lib.tmo_blocks.argtypes = [p64, i64, i64, p64, p64, i64]
        lib.tmo_blocks.restype = i64
        lib.tmo_copy.argtypes = [ctypes.c_int, p64, i64, pu8, i64, i64, i64, pu8, i64, i64, ctypes.c_int]
        lib.tmo_copy.restype = i64
        _lib = lib
    return _lib


def encode(t) -> np.ndarray:
    """Recipe (nested tuples) -> the prefix-order int64 array the C oracle parses."""
    out = []

    def rec(t):
        kind = t[0]
        out.append(_KIND[kind])
        if kind == "named":
            out.append(_NAMED_SIZE[t[1]])
            return
        if kind == "contiguous":
            out.append(t[1])
        elif kind in ("vector", "hvector"):
            out.extend(t[1:4])
        else:
            _, sizes, subs, starts, order, _old = t
            out.extend([len(sizes), 0 if order == "C" else 1, *sizes, *subs, *starts])
        rec(t[-1])

    rec(t)
    return np.asarray(out, dtype=np.int64)


def _enc_ptr(enc):
    return enc.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), enc.size


def measure(t):
    """(size, lb, ub) of one object."""
    enc = encode(t)
    s, lb, ub = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rc = _load().tmo_measure(*_enc_ptr(enc), ctypes.byref(s), ctypes.byref(lb), ctypes.byref(ub))
    if rc != 0:
        raise ValueError("bad recipe")
    return s.value, lb.value, ub.value


def size(t):
    return measure(t)[0]


def extent(t):
    _, lb, ub = measure(t)
    return ub - lb


def blocks(t, incount: int = 1):
    """The type map of `incount` objects as two int64 arrays (displacements, lengths)."""
    enc = encode(t)
    lib = _load()
    n = lib.tmo_blocks(*_enc_ptr(enc), incount, None, None, 0)
    if n < 0:
        raise ValueError("bad recipe")
    disp = np.empty(n, dtype=np.int64)
    length = np.empty(n, dtype=np.int64)
    p64 = ctypes.POINTER(ctypes.c_int64)
    lib.tmo_blocks(*_enc_ptr(enc), incount, disp.ctypes.data_as(p64), length.ctypes.data_as(p64), n)
    return disp, length


def _copy(direction, typed, origin, count, t, packed, position, nthreads):
    assert typed.dtype == np.uint8 and packed.dtype == np.uint8
    assert typed.flags.c_contiguous and packed.flags.c_contiguous
    enc = encode(t)
    rc = _load().tmo_copy(direction, *_enc_ptr(enc), typed.ctypes.data, typed.size, origin, count,
                          packed.ctypes.data, packed.size, position, nthreads)
    if rc == -1:
        raise ValueError("bad recipe")
    if rc == -2:
        raise ValueError("truncate")
    if rc == -3:
        raise IndexError("type map leaves the buffer")
    return rc


def pack(inbuf, origin, incount, t, outbuf, position, nthreads: int = 1) -> int:
    """MPI_Pack on host arrays (uint8, C-contiguous); returns the new position."""
    return _copy(0, inbuf, origin, incount, t, outbuf, position, nthreads)


def unpack(inbuf, position, outbuf, origin, outcount, t, nthreads: int = 1) -> int:
    """MPI_Unpack on host arrays; returns the new position."""
    return _copy(1, outbuf, origin, outcount, t, inbuf, position, nthreads)
