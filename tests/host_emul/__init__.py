"""Builds and wraps tests/host_emul/emul.cpp: the library's planner and kernel body
compiled for the host, run thread by thread under bounds checks.  Tests only."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(os.path.dirname(_HERE))
_CSRC = os.path.join(_ROOT, "paper_2012_14363_amd", "csrc")
_LIB = os.path.join(_HERE, "libtp_emul.so")
_SOURCES = [os.path.join(_HERE, "emul.cpp"), os.path.join(_CSRC, "plan.cpp")]
_lib = None


def build(force=True):
    deps = _SOURCES + [os.path.join(_CSRC, h) for h in ("plan.hpp", "tile_body.hpp", "fastdiv.hpp", "strided_block.hpp")]
    stale = not os.path.exists(_LIB) or any(os.path.getmtime(d) > os.path.getmtime(_LIB) for d in deps)
    if force or stale:
        subprocess.check_call(["g++", "-O2", "-g", "-std=c++20", "-Wall", "-Wextra", "-Wno-unknown-pragmas", "-fPIC",
                               "-shared", "-I", _CSRC, *_SOURCES, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        i64, p64, vp = ctypes.c_int64, ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p
        L.emul_transfer.argtypes = [ctypes.c_int, ctypes.c_int, i64, p64, p64, i64, i64, vp, i64, i64, vp, i64, i64,
                                    ctypes.c_int, i64, i64, ctypes.c_int, vp, p64, ctypes.c_char_p, i64]
        L.emul_transfer.restype = ctypes.c_int
        pint = ctypes.POINTER(ctypes.c_int)
        L.emul_transfer_batch.argtypes = [ctypes.c_int, ctypes.c_int, pint, p64, p64, p64, p64, p64, p64, p64, vp, i64,
                                          vp, i64, i64, vp, p64]
        L.emul_transfer_batch.restype = ctypes.c_int
        L.emul_fastdiv_mismatches.argtypes = [ctypes.c_uint32, i64, ctypes.c_uint64]
        L.emul_fastdiv_mismatches.restype = i64
        _lib = L
    return _lib


def fastdiv_mismatches(small_limit, random_pairs, seed):
    return _load().emul_fastdiv_mismatches(small_limit, random_pairs, seed)


def transfer(unpack, block, extent, count, typed, origin, packed, position, *, max_word=16,
             max_rows_per_launch=1 << 30, max_words_per_run=1 << 30, allow_shift=True, count_writes=True):
    """Emulates tp_pack / tp_unpack on host numpy uint8 arrays.

    `block` = (start, counts, strides) as returned by tp_type_get_strided_block.
    Returns a dict with the checks' tallies and the plan text."""
    start, counts, strides = block
    nd = len(counts)
    arr = ctypes.c_int64 * nd
    dst = typed if unpack else packed
    wc = np.zeros(dst.size, dtype=np.uint8) if count_writes else None
    result = (ctypes.c_int64 * 4)()
    text = ctypes.create_string_buffer(1 << 16)
    rc = _load().emul_transfer(int(unpack), nd, start, arr(*counts), arr(*strides), extent, count,
                               typed.ctypes.data, typed.size, origin, packed.ctypes.data, packed.size, position,
                               {1: 0, 2: 1, 4: 2, 8: 3, 16: 4}[max_word], max_rows_per_launch, max_words_per_run,
                               int(allow_shift),
                               wc.ctypes.data if wc is not None else None, result, text, len(text))
    return {"rc": rc, "oob": result[0], "misaligned": result[1], "rewritten": result[2], "launches": result[3],
            "plan": text.value.decode(), "write_count": wc}


def transfer_batch(unpack, requests, typed, packed, position, count_writes=True):
    """Emulates tp_pack_batch / tp_unpack_batch.  `requests` = list of dicts with keys
    block (start, counts, strides), extent, count, origin, size (bytes of one object)."""
    n = len(requests)
    ndims = (ctypes.c_int * n)(*[len(r["block"][1]) for r in requests])
    starts = (ctypes.c_int64 * n)(*[r["block"][0] for r in requests])
    counts = (ctypes.c_int64 * (16 * n))()
    strides = (ctypes.c_int64 * (16 * n))()
    for i, r in enumerate(requests):
        for d, (c, s) in enumerate(zip(r["block"][1], r["block"][2])):
            counts[16 * i + d], strides[16 * i + d] = c, s
    arr = lambda key: (ctypes.c_int64 * n)(*[r[key] for r in requests])  # noqa: E731
    dst = typed if unpack else packed
    wc = np.zeros(dst.size, dtype=np.uint8) if count_writes else None
    result = (ctypes.c_int64 * 5)()
    rc = _load().emul_transfer_batch(int(unpack), n, ndims, starts, counts, strides, arr("extent"), arr("count"),
                                     arr("origin"), arr("size"), typed.ctypes.data, typed.size,
                                     packed.ctypes.data, packed.size, position,
                                     wc.ctypes.data if wc is not None else None, result)
    return {"rc": rc, "oob": result[0], "misaligned": result[1], "rewritten": result[2], "batches": result[3],
            "singles": result[4], "write_count": wc}
