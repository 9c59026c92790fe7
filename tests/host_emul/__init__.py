"""Builds and wraps tests/host_emul/*.cpp: the library's planner and kernel body compiled for
the host and run thread by thread under bounds checks, and its resource cache and buffer map
over made-up memory.  Tests only."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(os.path.dirname(_HERE))
_CSRC = os.path.join(_ROOT, "paper_2012_14363_amd", "csrc")
# TP_SANITIZE=address (AddressSanitizer + UndefinedBehaviorSanitizer) or =thread (ThreadSanitizer) builds
# this library, and the C oracle, instrumented and under a name of its own; the process that loads it
# must have the sanitizer's runtime preloaded (README: "Sanitizer builds").  CPU only.
SANITIZE = os.environ.get("TP_SANITIZE", "")
SANITIZE_FLAGS = {"": [], "address": ["-fsanitize=address,undefined", "-fno-omit-frame-pointer"],
                  "thread": ["-fsanitize=thread", "-fno-omit-frame-pointer"]}[SANITIZE]
_LIB = os.path.join(_HERE, f"libtp_emul{'.' + SANITIZE if SANITIZE else ''}.so")
_SOURCES = [os.path.join(_HERE, "emul.cpp"), os.path.join(_HERE, "cache_emul.cpp"), os.path.join(_HERE, "types_emul.cpp"),
            os.path.join(_CSRC, "plan.cpp"), os.path.join(_CSRC, "resource_cache.cpp"), os.path.join(_CSRC, "type_tree.cpp"),
            os.path.join(_CSRC, "canon.cpp")]
_lib = None


def build(force=True):
    deps = _SOURCES + [os.path.join(_CSRC, h) for h in ("plan.hpp", "tile_body.hpp", "fastdiv.hpp", "strided_block.hpp",
                                                         "resource_cache.hpp", "buffer_map.hpp", "type_tree.hpp", "canon.hpp")]
    stale = not os.path.exists(_LIB) or any(os.path.getmtime(d) > os.path.getmtime(_LIB) for d in deps)
    if force or stale:
        subprocess.check_call(["g++", "-O2", "-g", "-std=c++20", "-Wall", "-Wextra", "-Wno-unknown-pragmas", "-fPIC",
                               "-shared", "-pthread", *SANITIZE_FLAGS, "-I", _CSRC, *_SOURCES, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        i64, p64, vp = ctypes.c_int64, ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p
        L.emul_transfer.argtypes = [ctypes.c_int, ctypes.c_int, i64, p64, p64, i64, i64, vp, i64, i64, vp, i64, i64,
                                    ctypes.c_int, i64, i64, ctypes.c_int, ctypes.c_int, i64, vp, p64, ctypes.c_char_p, i64]
        L.emul_transfer.restype = ctypes.c_int
        pint = ctypes.POINTER(ctypes.c_int)
        L.emul_transfer_batch.argtypes = [ctypes.c_int, ctypes.c_int, pint, p64, p64, p64, p64, p64, p64, p64, vp, i64,
                                          vp, i64, i64, vp, p64]
        L.emul_transfer_batch.restype = ctypes.c_int
        L.emul_plan_only.argtypes = [ctypes.c_int, ctypes.c_int, i64, p64, p64, i64, i64, i64, i64, ctypes.c_int, p64, i64]
        L.emul_plan_only.restype = i64
        L.types_emul_hammer.argtypes = [ctypes.c_int, ctypes.c_int]
        L.types_emul_hammer.restype = i64
        L.emul_fastdiv_mismatches.argtypes = [ctypes.c_uint32, i64, ctypes.c_uint64]
        L.emul_fastdiv_mismatches.restype = i64
        L.cache_emul_new.restype = vp
        L.cache_emul_delete.argtypes = [vp]
        L.cache_emul_acquire.argtypes = [vp, ctypes.c_int, i64, ctypes.POINTER(vp)]
        L.cache_emul_release.argtypes = [vp, ctypes.c_int, vp]
        L.cache_emul_trim.argtypes = [vp]
        L.cache_emul_trim.restype = i64
        L.cache_emul_counts.argtypes = [vp, ctypes.c_int, p64]
        L.cache_emul_find.argtypes = [vp, vp, pint, p64, p64]
        L.cache_emul_capacity.argtypes = [i64]
        L.cache_emul_capacity.restype = i64
        L.cache_emul_backend.argtypes = [ctypes.c_int, p64]
        L.cache_emul_hammer.argtypes = [vp, ctypes.c_int, ctypes.c_int]
        L.cache_emul_hammer.restype = i64
        L.bufmap_emul_run.argtypes = [ctypes.c_int, p64, p64, pint, ctypes.c_int, ctypes.c_int, ctypes.c_int, p64, pint,
                                      pint, p64]
        L.bufmap_emul_run.restype = i64
        _lib = L
    return _lib


def buffer_map_run(allocations, ops, bounds_known=True, checked=True):
    """One BufferMap against made-up allocations [(lo, hi, is_host)], locating ops [(address,
    allow_host)] in order.  Returns (queries made, [(status, view - address)])."""
    na, no = len(allocations), len(ops)
    lo = (ctypes.c_int64 * na)(*[a[0] for a in allocations])
    hi = (ctypes.c_int64 * na)(*[a[1] for a in allocations])
    host = (ctypes.c_int * na)(*[int(a[2]) for a in allocations])
    addr = (ctypes.c_int64 * no)(*[o[0] for o in ops])
    allow = (ctypes.c_int * no)(*[int(o[1]) for o in ops])
    status = (ctypes.c_int * no)()
    delta = (ctypes.c_int64 * no)()
    q = _load().bufmap_emul_run(na, lo, hi, host, int(bounds_known), int(checked), no, addr, allow, status, delta)
    return q, list(zip(status, delta))


COUNT_FIELDS = ("hits", "misses", "idle", "leased", "idle_bytes", "leased_bytes")


class Cache:
    """The library's ResourceCache over the host heap (cache_emul.cpp)."""

    def __init__(self):
        self._L = _load()
        self._c = self._L.cache_emul_new()

    def close(self):
        if self._c:
            self._L.cache_emul_delete(self._c)
            self._c = None

    def acquire(self, kind, nbytes):
        """(status, handle address or None)"""
        h = ctypes.c_void_p()
        rc = self._L.cache_emul_acquire(self._c, kind, nbytes, ctypes.byref(h))
        return rc, h.value

    def release(self, kind, handle):
        return self._L.cache_emul_release(self._c, kind, handle)

    def trim(self):
        return self._L.cache_emul_trim(self._c)

    def counts(self, kind):
        out = (ctypes.c_int64 * 6)()
        self._L.cache_emul_counts(self._c, kind, out)
        return dict(zip(COUNT_FIELDS, out))

    def find(self, address):
        """None, or (kind, gpu view minus address, bytes to the buffer's end)."""
        kind, delta, room = ctypes.c_int(), ctypes.c_int64(), ctypes.c_int64()
        if not self._L.cache_emul_find(self._c, address, ctypes.byref(kind), ctypes.byref(delta), ctypes.byref(room)):
            return None
        return kind.value, delta.value, room.value

    def hammer(self, threads, rounds):
        return self._L.cache_emul_hammer(self._c, threads, rounds)


def cache_capacity(nbytes):
    return _load().cache_emul_capacity(nbytes)


def cache_backend(kind):
    """Backend tallies: (created, destroyed) of `kind`, live buffer bytes of all kinds."""
    out = (ctypes.c_int64 * 3)()
    _load().cache_emul_backend(kind, out)
    return tuple(out)


def cache_fail_next(n):
    _load().cache_emul_fail_next(n)


def cache_set_device(d):
    _load().cache_emul_set_device(d)


def types_hammer(threads, rounds):
    """Threads building, committing, looking up and freeing datatypes through the library's handle table
    (types_emul.cpp); returns the number of wrong results."""
    return _load().types_emul_hammer(threads, rounds)


def fastdiv_mismatches(small_limit, random_pairs, seed):
    return _load().emul_fastdiv_mismatches(small_limit, random_pairs, seed)


def transfer(unpack, block, extent, count, typed, origin, packed, position, *, max_word=16,
             max_rows_per_launch=1 << 30, max_words_per_run=1 << 30, allow_xpose=True, stage=-1, stage_bytes=0,
             count_writes=True):
    """Emulates tp_pack / tp_unpack on host numpy uint8 arrays.

    `block` = (start, counts, strides) as returned by tp_type_get_strided_block.
    Returns a dict with the checks' tallies and the plan text."""
    start, counts, strides = block
    nd = len(counts)
    arr = ctypes.c_int64 * nd
    dst = typed if unpack else packed
    wc = np.zeros(dst.size, dtype=np.uint8) if count_writes else None
    result = (ctypes.c_int64 * 7)()
    text = ctypes.create_string_buffer(1 << 16)
    rc = _load().emul_transfer(int(unpack), nd, start, arr(*counts), arr(*strides), extent, count,
                               typed.ctypes.data, typed.size, origin, packed.ctypes.data, packed.size, position,
                               {1: 0, 2: 1, 4: 2, 8: 3, 16: 4}[max_word], max_rows_per_launch, max_words_per_run,
                               int(allow_xpose), stage, stage_bytes, wc.ctypes.data if wc is not None else None, result,
                               text, len(text))
    return {"rc": rc, "oob": result[0], "unaligned": result[1], "rewritten": result[2], "launches": result[3],
            "duplicates": result[4], "prefetched_span": result[5], "misplaced": result[6], "plan": text.value.decode(),
            "write_count": wc}


def plan_only(unpack, block, extent, count, typed_address=1 << 40, packed_address=1 << 44, batched=False):
    """Plans tp_pack / tp_unpack of a block at made-up addresses without touching memory.  Returns the
    launches as dicts (tiles, grid = workgroups asked for, rows, kind: 0 tile, 1 transposing, 2 read-only
    pass, 100 batched)."""
    start, counts, strides = block
    nd = len(counts)
    arr = ctypes.c_int64 * nd
    cap = 1 << 16
    out = (ctypes.c_int64 * (4 * cap))()
    n = _load().emul_plan_only(int(unpack), nd, start, arr(*counts), arr(*strides), extent, count, typed_address,
                               packed_address, int(batched), out, cap)
    if n < 0:
        raise ValueError(f"planner status {-n}")
    assert n <= cap
    return [dict(zip(("tiles", "grid", "rows", "kind"), out[4 * i:4 * i + 4])) for i in range(n)]


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
    result = (ctypes.c_int64 * 6)()
    rc = _load().emul_transfer_batch(int(unpack), n, ndims, starts, counts, strides, arr("extent"), arr("count"),
                                     arr("origin"), arr("size"), typed.ctypes.data, typed.size,
                                     packed.ctypes.data, packed.size, position,
                                     wc.ctypes.data if wc is not None else None, result)
    return {"rc": rc, "oob": result[0], "unaligned": result[1], "rewritten": result[2], "batches": result[3],
            "singles": result[4], "duplicates": result[5], "write_count": wc}
