"""CPU-only tests of the library's host logic: type sizes/bounds, canonicalization
(paper Sec. 3.1-3.3) against the oracle's type map, the C ABI's error behaviour and
exported symbols, and the planner + kernel body emulated on the host under bounds
checks.  No GPU compute call is made here."""
import ctypes
import os
import random
import re
import sys

import numpy as np
import pytest

import workloads as W
from workloads import BYTE, DOUBLE, FLOAT, contiguous, hvector, named, subarray, vector
from oracle import typemap as py
from oracle import typemap_c as cc
from paper_2012_14363_amd import binding as tp

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import host_emul  # noqa: E402

INT16 = named("INT16")


def expand(block, count=1, extent=0):
    """Byte displacements a StridedBlock selects, row-major over counts (last dim slowest)."""
    start, counts, strides = block
    out = []

    def rec(d, base):
        if d == 0:
            out.extend(range(base, base + counts[0]))
            return
        for i in range(counts[d]):
            rec(d - 1, base + i * strides[d])

    for obj in range(count):
        rec(len(counts) - 1, start + obj * extent)
    return out


# ------------------------------------------------------------------ ABI surface
def test_library_exports_every_declared_symbol():
    header = open(os.path.join(os.path.dirname(tp.LIB_PATH), "..", "include", "tp_pack.h")).read()
    declared = set(re.findall(r"\b(tp_[a-z_0-9]+)\s*\(", header))
    assert declared == set(tp.EXPORTS)
    lib = tp.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_predefined_types():
    for name, h in tp.PREDEFINED.items():
        assert tp.type_size(h) == py.NAMED_SIZE[name]
        assert tp.type_get_extent(h) == (0, py.NAMED_SIZE[name])
        assert tp.type_get_strided_block(h) == (0, [py.NAMED_SIZE[name]], [1])


# ------------------------------------------------------------------ canonical forms
def test_config_canonical_forms():
    b = lambda r: tp.type_get_strided_block(tp.type_from_recipe(r))  # noqa: E731
    # 2D vector: both constructions give the same block
    for r in W.configs.cfg1()["recipes"].values():
        assert b(r) == (0, [8, 64], [1, 512])
    # 3D strided block: generic, flattened (a1 = 512), dense-folded (a0 = 512), fully dense
    assert b(W.configs.cfg2_point(16, 1 << 20)["recipe"]) == (0, [16, 256, 256], [1, 512, 262144])
    assert b(W.configs.cfg2_point(4, 1 << 20)["recipe"]) == (0, [4, 1 << 18], [1, 512])
    assert b(W.configs.cfg2_point(512, 1 << 20)["recipe"]) == (0, [32768, 32], [1, 262144])
    assert b(W.configs.cfg2_point(512, 1 << 26)["recipe"]) == (0, [1 << 26], [1])
    # halo: the 8-byte element folds into the x run; nothing else merges
    c3 = W.configs.cfg3()
    shapes = set()
    for r, reg in zip(c3["send"], c3["send_region"]):
        start, counts, strides = b(r)
        (z0, z1), (y0, y1), (x0, x1) = reg
        assert start == ((z0 * 512 + y0) * 512 + x0) * 8
        assert counts == [8 * (x1 - x0), y1 - y0, z1 - z0] and strides == [1, 4096, 2097152]
        shapes.add(tuple(counts))
    assert shapes == {(24, 506, 506), (4048, 3, 506), (4048, 506, 3), (4048, 3, 3), (24, 506, 3), (24, 3, 506),
                      (24, 3, 3)}
    # tiny runs
    assert b(W.configs.cfg4_point(3)["recipe"]) == (0, [3, 1 << 24], [1, 64])
    assert b(W.configs.cfg4_point(3)["recipe_subarray"](5)) == (5, [3, 1 << 24], [1, 64])
    # 4-level nested type: 4D, strides not monotone because nesting order is kept
    t5 = tp.type_from_recipe(W.configs.cfg5()["recipe"])
    assert tp.type_get_strided_block(t5) == (50432, [4096, 8, 16, 4], [1, 16384, 8192, 2342912])
    assert tp.type_size(t5) == 2097152 and tp.type_get_extent(t5) == (0, 8200192)


def test_each_pass_on_its_own():
    b = lambda r: tp.type_get_strided_block(tp.type_from_recipe(r))  # noqa: E731
    # dense folding (Alg. 2): a stream of abutting dense elements is one dense run
    assert b(contiguous(10, FLOAT)) == (0, [40], [1])
    assert b(vector(5, 4, 4, BYTE)) == (0, [20], [1])
    # ... but not when the oldtype has holes: contiguous(3, {0,2}) stays strided
    assert b(contiguous(3, vector(2, 1, 2, BYTE))) == (0, [1, 2, 3], [1, 2, 3])
    # stream elision (Alg. 3): count-1 streams vanish, their offsets survive
    assert b(hvector(1, 1, 9999, vector(4, 2, 8, BYTE))) == b(vector(4, 2, 8, BYTE)) == (0, [2, 4], [1, 8])
    assert b(subarray((7, 9), (1, 3), (2, 4), "C", BYTE)) == (2 * 9 + 4, [3], [1])
    # stream flattening (Alg. 4): rows whose pitch continues the inner stream
    assert b(hvector(6, 1, 40, hvector(5, 1, 8, INT16))) == (0, [2, 30], [1, 8])
    # the paper's worked sizes (Sec. 3.1 figure caption): 100 x 13 x 47 bytes in 256 x 512 x 1024
    assert b(subarray((1024, 512, 256), (47, 13, 100), (0, 0, 0), "C", BYTE)) == (0, [100, 13, 47], [1, 256, 131072])
    assert b(hvector(47, 1, 256 * 512, vector(13, 100, 256, BYTE))) == (0, [100, 13, 47], [1, 256, 131072])
    # ... and with FLOAT elements and the row pitch counted in elements
    assert b(subarray((1024, 512, 256), (47, 13, 100), (0, 0, 0), "C", FLOAT)) == (0, [400, 13, 47],
                                                                                    [1, 1024, 524288])
    # Fortran order reverses which dimension is contiguous
    assert b(subarray((256, 512, 1024), (100, 13, 47), (0, 0, 0), "F", BYTE)) == (0, [100, 13, 47], [1, 256, 131072])
    # nesting order is kept: same byte set, other order, other block
    assert b(hvector(3, 1, 8, hvector(2, 1, 2, BYTE))) == (0, [1, 2, 3], [1, 2, 8])
    assert b(hvector(2, 1, 2, hvector(3, 1, 8, BYTE))) == (0, [1, 3, 2], [1, 8, 2])
    # empty types
    assert b(vector(0, 2, 4, BYTE)) == (0, [0], [1])
    assert b(subarray((4, 6), (2, 0), (1, 2), "C", BYTE)) == (0, [0], [1])


def _equivalent_cuboids(e, a):
    from test_oracle_pins import _cuboids
    return _cuboids(e, a)


def test_paper_equivalent_constructions_share_one_block():
    blocks = {str(tp.type_get_strided_block(tp.type_from_recipe(t))) for t in _equivalent_cuboids((5, 3, 4), (8, 6, 5))}
    assert blocks == {str((0, [20, 3, 4], [1, 32, 192]))}


def _random_types(seed, n, **kw):
    rng = random.Random(seed)
    out = []
    while len(out) < n:
        t = W.random_recipe(rng, rng.randint(1, 4), **kw)
        if py.size(t) <= 2048:
            out.append(t)
    return out


def test_canonical_block_expands_to_the_oracle_type_map():
    # what pins the canonicalizer: for thousands of random trees (negative strides, zero counts,
    # self-overlap included) the StridedBlock enumerates exactly the oracle's byte sequence
    seen = {}
    for t in _random_types(201, 3000, allow_negative=True, allow_zero=True, allow_overlap=True):
        h = tp.type_from_recipe(t)
        block = tp.type_get_strided_block(h)
        disp = py.byte_displacements(t)
        assert expand(block) == disp, t
        assert tp.type_size(h) == py.size(t), t
        lb, ub = py.bounds(t)
        assert tp.type_get_extent(h) == (lb, ub - lb), t
        key = tuple(disp)
        if not py.has_overlap(t) and disp:
            # identical ordered type maps must give the identical block
            assert seen.setdefault(key, block) == block, t
        if h >= 12:
            tp.type_free(h)
    assert len(seen) > 300


def test_incount_objects_follow_extent():
    for t in _random_types(202, 200, allow_negative=True):
        h = tp.type_from_recipe(t)
        ex = tp.type_get_extent(h)[1]
        assert expand(tp.type_get_strided_block(h), 3, ex) == py.byte_displacements(t, 3)
        assert tp.pack_size(3, h) == 3 * py.size(t)


# ------------------------------------------------------------------ error behaviour
def test_error_codes_and_unchanged_outputs():
    L = tp.lib()
    new = ctypes.c_int32(777)
    assert L.tp_type_contiguous(-1, tp.TP_BYTE, ctypes.byref(new)) == tp.TP_ERR_COUNT
    assert L.tp_type_vector(2, -3, 1, tp.TP_BYTE, ctypes.byref(new)) == tp.TP_ERR_COUNT
    assert L.tp_type_contiguous(2, 12345678, ctypes.byref(new)) == tp.TP_ERR_TYPE
    assert L.tp_type_contiguous(2, -5, ctypes.byref(new)) == tp.TP_ERR_TYPE
    assert L.tp_type_contiguous(2, tp.TP_BYTE, None) == tp.TP_ERR_ARG
    arr = ctypes.c_int * 2
    sub = L.tp_type_create_subarray
    assert sub(2, arr(4, 6), arr(5, 1), arr(0, 0), 0, tp.TP_BYTE, ctypes.byref(new)) == tp.TP_ERR_ARG
    assert sub(2, arr(4, 6), arr(2, 3), arr(3, 0), 0, tp.TP_BYTE, ctypes.byref(new)) == tp.TP_ERR_ARG
    assert sub(2, arr(4, 6), arr(2, 3), arr(0, 0), 7, tp.TP_BYTE, ctypes.byref(new)) == tp.TP_ERR_ARG
    assert sub(0, arr(4, 6), arr(2, 3), arr(0, 0), 0, tp.TP_BYTE, ctypes.byref(new)) == tp.TP_ERR_ARG
    assert sub(2, arr(4, 6), arr(2, -3), arr(0, 0), 0, tp.TP_BYTE, ctypes.byref(new)) == tp.TP_ERR_ARG
    big = ctypes.c_int32()
    assert L.tp_type_vector(2 ** 31 - 1, 2 ** 31 - 1, 2 ** 31 - 1, tp.TP_BYTE, ctypes.byref(big)) == tp.TP_SUCCESS
    assert L.tp_type_vector(2 ** 31 - 1, 2 ** 31 - 1, 1, big, ctypes.byref(new)) == tp.TP_ERR_RANGE
    assert new.value == 777

    t = tp.type_vector(3, 2, 4, tp.TP_BYTE)
    pos = ctypes.c_int64(5)
    fake = ctypes.c_void_p(4096)
    # not committed yet
    assert L.tp_pack(fake, 1, t, fake, 100, ctypes.byref(pos), None) == tp.TP_ERR_TYPE
    nd, st = ctypes.c_int(), ctypes.c_int64()
    c16 = (ctypes.c_int64 * 16)()
    assert L.tp_type_get_strided_block(t, ctypes.byref(nd), ctypes.byref(st), c16, c16) == tp.TP_ERR_TYPE
    tp.type_commit(t)
    tp.type_commit(t)  # idempotent
    assert L.tp_pack(fake, -1, t, fake, 100, ctypes.byref(pos), None) == tp.TP_ERR_COUNT
    assert L.tp_pack(fake, 1, t, fake, 10, ctypes.byref(pos), None) == tp.TP_ERR_TRUNCATE   # 5 + 6 > 10
    assert L.tp_unpack(fake, 10, ctypes.byref(pos), fake, 1, t, None) == tp.TP_ERR_TRUNCATE
    assert L.tp_pack(None, 1, t, fake, 100, ctypes.byref(pos), None) == tp.TP_ERR_BUFFER
    assert L.tp_pack(fake, 1, t, None, 100, ctypes.byref(pos), None) == tp.TP_ERR_BUFFER
    assert L.tp_pack(fake, 1, t, fake, 100, None, None) == tp.TP_ERR_ARG
    neg = ctypes.c_int64(-1)
    assert L.tp_pack(fake, 1, t, fake, 100, ctypes.byref(neg), None) == tp.TP_ERR_ARG
    assert pos.value == 5 and neg.value == -1
    # zero objects: a successful no-op that needs no buffers and no device
    assert L.tp_pack(None, 0, t, None, 0, ctypes.byref(ctypes.c_int64(0)), None) == tp.TP_SUCCESS
    empty = tp.type_from_recipe(vector(0, 2, 4, BYTE))
    assert L.tp_pack(None, 5, empty, None, 0, ctypes.byref(ctypes.c_int64(0)), None) == tp.TP_SUCCESS

    h = ctypes.c_int32(t)
    assert L.tp_type_free(ctypes.byref(h)) == tp.TP_SUCCESS and h.value == tp.TP_TYPE_NULL
    assert L.tp_type_size(t, ctypes.byref(ctypes.c_int64())) == tp.TP_ERR_TYPE        # stale handle
    assert L.tp_type_free(ctypes.byref(ctypes.c_int32(tp.TP_BYTE))) == tp.TP_ERR_TYPE  # predefined
    assert L.tp_set_override(b"no_such_key", b"1") == tp.TP_ERR_ARG
    assert L.tp_set_override(b"word", b"3") == tp.TP_ERR_ARG
    for code in range(0, 9):
        assert tp.error_string(code)


def test_freeing_the_oldtype_keeps_the_derived_type_alive():
    row = tp.type_contiguous(8, tp.TP_BYTE)
    plane = tp.type_create_hvector(64, 1, 512, row)
    tp.type_free(row)
    tp.type_commit(plane)
    assert tp.type_get_strided_block(plane) == (0, [8, 64], [1, 512])
    # a recycled slot must not resurrect the stale handle
    other = tp.type_contiguous(3, tp.TP_BYTE)
    with pytest.raises(tp.TpError):
        tp.type_size(row)
    tp.type_free(other)
    tp.type_free(plane)


# ------------------------------------------- planner + kernel body, emulated on the host
def _emulate_roundtrip(t, incount, *, typed_shift=0, packed_shift=0, position=0, **kw):
    h = tp.type_from_recipe(t)
    block = tp.type_get_strided_block(h)
    lb, ex = tp.type_get_extent(h)
    size = tp.type_size(h) * incount
    # a subarray's bounds are those of the full array even when its oldtype reaches below its
    # origin, so size the buffer from the bytes actually selected
    disps = py.byte_displacements(t, incount)
    lo, hi = min(0, min(disps)), max(0, max(disps) + 1)
    pad = 32
    origin = -lo + pad + typed_shift
    n = hi - lo + 2 * pad + typed_shift
    rng = np.random.default_rng(hash((str(t), incount)) & 0xFFFFFFFF)
    typed_store = np.zeros(n + 128, dtype=np.uint8)
    base = (-typed_store.ctypes.data) % 128         # 128-byte aligned window, then shifted
    typed = typed_store[base:base + n]
    typed[:] = rng.integers(0, 256, n, dtype=np.uint8)
    packed_store = np.zeros(size + position + 64 + 16, dtype=np.uint8)
    pbase = (-packed_store.ctypes.data) % 64 + packed_shift
    packed = packed_store[pbase:pbase + position + size]
    packed[:] = 0xEE

    res = host_emul.transfer(False, block, ex, incount, typed, origin, packed, position, **kw)
    assert res["rc"] == 0 and res["oob"] == 0 and res["rewritten"] == 0, (t, res)
    expect = np.full(position + size, 0xEE, dtype=np.uint8)
    assert cc.pack(typed, origin, incount, t, expect, position) == position + size
    assert np.array_equal(packed, expect), (t, res["plan"])
    # every packed byte is written; only where the last word of a run overlaps its neighbour
    # (at most W - 1 < 16 bytes per run or run piece) is a byte written twice, with the same value
    wc = res["write_count"]
    assert (wc[position:] >= 1).all() and (wc[:position] == 0).all()
    assert res["duplicates"] == int(wc.sum()) - size
    runs = size // max(1, block[1][0]) * (1 + block[1][0] // max(1, kw.get("max_words_per_run", 1 << 30)))
    assert res["duplicates"] <= 15 * max(runs, 1), (t, res)

    if not py.has_overlap(t, incount):
        dst_store = np.zeros(n + 128, dtype=np.uint8)
        dbase = (-dst_store.ctypes.data) % 128     # aligned like the buffer that was packed from
        dst = dst_store[dbase:dbase + n]
        dst[:] = 0xA5
        back = host_emul.transfer(True, block, ex, incount, dst, origin, packed, position, **kw)
        assert back["rc"] == 0 and back["oob"] == 0 and back["rewritten"] == 0, (t, back)
        # staged unpack: every store pass reads its packed bytes from the tile of the same index of the read-only pass
        assert back["misplaced"] == 0, (t, back["plan"])
        want = np.full(n, 0xA5, dtype=np.uint8)
        cc.unpack(packed, position, want, origin, incount, t)
        assert np.array_equal(dst, want), (t, back["plan"])
        res["unpack_plan"] = back["plan"]
        res["unpack_prefetched_span"] = back["prefetched_span"]
        res["unpack_compared"] = True
    if h >= 12:
        tp.type_free(h)
    return res


def test_emulated_kernels_match_oracle_on_random_types():
    rng = random.Random(303)
    compared = 0
    for i, t in enumerate(_random_types(301, 250, allow_negative=True, allow_zero=False)):
        res = _emulate_roundtrip(t, rng.randint(1, 3), typed_shift=rng.choice((0, 0, 1, 2, 4, 8)),
                                 packed_shift=rng.choice((0, 0, 1, 2, 4, 8)), position=rng.choice((0, 3, 16)),
                                 stage=rng.choice((-1, 1)), stage_bytes=rng.choice((0, 4096)))
        compared += bool(res.get("unpack_compared"))
    # types whose map overlaps itself have no unique unpack and are only packed: they must stay the exception
    assert compared >= 200, compared


@pytest.mark.parametrize("a0", [1, 2, 4, 8, 16, 48, 64, 200, 512, 1040, 4100, 4112])
def test_emulated_tile_shapes(a0):
    # run lengths that exercise every (ux, ur) tile and ragged tails, 2D and 3D
    _emulate_roundtrip(hvector(3, 1, 5 * 8192, hvector(5, 1, 8192, contiguous(a0, BYTE))), 2)
    _emulate_roundtrip(vector(37, a0, a0 + 16, BYTE), 1)


def test_emulated_word_width_follows_run_length_only():
    # 16-byte words wherever a run holds 16 bytes, at any address and for any run length or stride
    t = vector(16, 64, 128, BYTE)
    for shift in (0, 8, 4, 2, 1, 3, 7):
        for kw in ({"typed_shift": shift}, {"packed_shift": shift}, {"position": shift}):
            res = _emulate_roundtrip(t, 1, **kw)
            assert "tile W=16 " in res["plan"] and "n0=4 back=0 " in res["plan"]
            assert (res["unaligned"] > 0) == (shift % 16 != 0) and res["duplicates"] == 0
    # unpack: rows made of whole aligned 128-byte lines keep 16-byte words, four rows per thread and
    # plain streaming stores (the helper puts the origin 32 bytes into a 128-byte aligned window)
    full = vector(16, 128, 256, BYTE)
    assert "tile W=16 ux=1 ur=4 nt=3 " in _emulate_roundtrip(full, 1, typed_shift=96)["unpack_plan"]
    assert "tile W=16 ux=1 ur=4 nt=3 " in _emulate_roundtrip(full, 1, typed_shift=96, position=7, packed_shift=1)["unpack_plan"]
    assert "tile W=16 ux=1 ur=1 nt=7 " in _emulate_roundtrip(full, 1, typed_shift=32)["unpack_plan"]       # rows start mid-line
    assert "tile W=8 ux=1 ur=1 nt=7 " in _emulate_roundtrip(t, 1, typed_shift=96)["unpack_plan"]             # half lines
    # all other rows, if closer together than a page: written through, one row per thread, 8 to 15 lanes per row
    assert "tile W=8 ux=1 ur=1 nt=7 bx=8 n0=8 " in _emulate_roundtrip(t, 1, typed_shift=16)["unpack_plan"]
    assert "tile W=8 ux=1 ur=1 nt=7 " in _emulate_roundtrip(vector(16, 64, 96, BYTE), 1, typed_shift=32)["unpack_plan"]   # stride 96
    res = _emulate_roundtrip(vector(16, 200, 512, BYTE), 1)
    assert "W=16 " in res["plan"] and "W=16 ux=1 ur=1 nt=7 bx=16 n0=13 back=8" in res["unpack_plan"]
    res = _emulate_roundtrip(vector(16, 201, 512, BYTE), 1, typed_shift=3)
    assert "W=16 " in res["plan"] and "W=16 ux=1 ur=1 nt=7 bx=16 n0=13 back=7" in res["unpack_plan"]
    wt = lambda n, **kw: _emulate_roundtrip(vector(16, n, 128, BYTE), 1, **kw)["unpack_plan"]  # noqa: E731
    assert "W=8 ux=1 ur=1 nt=7 bx=16 n0=13 back=4 " in wt(100) and "W=4 ux=1 ur=1 nt=7 bx=8 n0=8 " in wt(32)
    assert "W=2 ux=1 ur=1 nt=7 bx=16 n0=12 " in wt(24) and "W=2 ux=1 ur=1 nt=7 bx=8 n0=8 " in wt(16)
    assert "W=1 ux=1 ur=1 nt=7 bx=16 n0=12 " in wt(12) and "W=1 ux=1 ur=1 nt=7 bx=8 n0=8 " in wt(8)
    assert "W=1 ux=1 ur=1 nt=7 bx=4 n0=3 " in wt(3, typed_shift=5) and "W=1 ux=1 ur=1 nt=7 bx=1 n0=1 " in wt(1)
    # rows a page or more apart keep the narrow words, four rows per thread and plain streaming stores
    assert "W=4 ux=1 ur=4 nt=3 bx=64 n0=50 " in _emulate_roundtrip(vector(16, 200, 4096, BYTE), 1)["unpack_plan"]
    assert "W=8 ux=1 ur=4 nt=3 " in _emulate_roundtrip(vector(5, 1040, 8192, BYTE), 1)["unpack_plan"]
    assert "W=16 ux=1 ur=1 nt=7 bx=256 n0=129 back=8 " in _emulate_roundtrip(vector(5, 2056, 2100, BYTE), 1)["unpack_plan"]
    assert "W=16 " in _emulate_roundtrip(contiguous(4099, BYTE), 1, typed_shift=1)["unpack_plan"]  # one run: no rows
    assert "W=4 " in _emulate_roundtrip(t, 1, max_word=4)["plan"]
    assert "W=16 bx=4 n0=3 back=0 " in _emulate_roundtrip(vector(16, 48, 64, BYTE), 1)["plan"].replace("ux=1 ur=4 nt=3 ", "")
    # 40 bytes = two whole words and a third pulled back by 8; the overlap is written twice
    res = _emulate_roundtrip(vector(16, 40, 64, BYTE), 1)
    assert "W=16 " in res["plan"] and "n0=3 back=8 " in res["plan"] and res["duplicates"] == 16 * 8
    assert "W=16 " in _emulate_roundtrip(vector(16, 36, 38, BYTE), 1)["plan"]          # stride 38
    assert "W=16 " in _emulate_roundtrip(vector(2, 16, 17, FLOAT), 3)["plan"]          # extent 132
    assert "W=16 " in _emulate_roundtrip(vector(9, 67, 71, BYTE), 1, typed_shift=1)["plan"]
    # a run shorter than 16 bytes that is the whole message: the largest power of two it holds
    assert "W=8 " in _emulate_roundtrip(contiguous(13, BYTE), 1)["plan"]
    assert "W=2 " in _emulate_roundtrip(contiguous(3, BYTE), 1, typed_shift=1)["plan"]
    # runs of at most 32 bytes: at least four lanes per row and at most 4-byte words
    short = lambda n, **kw: _emulate_roundtrip(vector(16, n, 64, BYTE), 1, **kw)["plan"].replace("ux=1 ur=4 nt=3 ", "")  # noqa: E731
    assert "W=4 bx=8 " in short(32) and "W=4 bx=4 " in short(16) and "W=2 bx=4 " in short(8)
    assert "W=1 bx=4 " in short(4) and "W=1 bx=2 " in short(2) and "W=1 bx=1 " in short(1)
    assert "W=4 bx=8 n0=6 back=0 " in short(24) and "W=2 bx=8 n0=6 back=0 " in short(12)
    assert "W=4 bx=8 n0=6 back=0 " in short(24, typed_shift=1, packed_shift=3)      # whatever the addresses
    assert "W=4 bx=8 n0=7 back=3 " in short(25) and "W=1 bx=4 n0=3 " in short(3)
    assert "W=16 bx=4 n0=3 back=15 " in short(33)


def test_emulated_staged_unpack_of_tiny_rows():
    # rows of one word at a pitch of 512, 256 or 128 bytes: chunks of packed bytes, each a read-only pass
    # followed by store passes whose rows are 512 bytes apart, all with the same few workgroups
    res = _emulate_roundtrip(vector(5000, 1, 512, BYTE), 1, stage=1, stage_bytes=4096)
    lines = res["unpack_plan"].splitlines()
    assert lines[0] == "prefetch bytes=4096 tile=256 blocks=16 grid=16", lines
    assert lines[1] == "tile W=1 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=4096 nrd=1 blocks=16 grid=16", lines
    assert lines[2] == "prefetch bytes=904 tile=256 blocks=4 grid=4" and " rows=904 " in lines[3] and len(lines) == 4, lines
    assert res["unpack_prefetched_span"] == 5000 and "prefetch" not in res["plan"]
    # four passes over every fourth row at 128-byte pitch; the packed rows of a pass are four words apart
    res = _emulate_roundtrip(vector(12001, 1, 128, BYTE), 1, stage=1, stage_bytes=8192, typed_shift=3, position=5)
    lines = res["unpack_plan"].splitlines()
    assert lines[0] == "prefetch bytes=8192 tile=1024 blocks=8 grid=8", lines
    assert [ln.split(" bx")[0] for ln in lines[1:5]] == ["tile W=1 ux=1 ur=1 nt=6"] * 4 and all(" rows=2048 " in ln for ln in lines[1:5])
    assert lines[5] == "prefetch bytes=3809 tile=1024 blocks=4 grid=4", lines
    assert [int(ln.split("rows=")[1].split()[0]) for ln in lines[6:]] == [953, 952, 952, 952], lines
    assert res["unpack_prefetched_span"] == 12001
    # two passes at 256-byte pitch, 4-byte rows, odd addresses on both sides (a chunk is one tile of both passes at least)
    res = _emulate_roundtrip(vector(2700, 4, 256, BYTE), 1, stage=1, stage_bytes=4096, typed_shift=1, packed_shift=3, position=2)
    assert res["unpack_plan"].count("prefetch") == 3 and res["unpack_plan"].count("tile W=4 ux=1 ur=1 nt=6") == 6
    res = _emulate_roundtrip(hvector(300, 1, -512, contiguous(2, BYTE)), 1, stage=1, stage_bytes=4096)     # negative pitch
    assert "prefetch" in res["unpack_plan"] and "tile W=2 ux=1 ur=1 nt=6" in res["unpack_plan"]
    # a last chunk of fewer than 16 bytes goes without its read-only pass; fewer rows than passes
    res = _emulate_roundtrip(vector(4101, 1, 512, BYTE), 1, stage=1, stage_bytes=4096)
    assert res["unpack_plan"].count("prefetch") == 1 and res["unpack_plan"].count("tile W=1") == 2
    res = _emulate_roundtrip(vector(3, 1, 128, BYTE), 1, stage=1)
    assert "prefetch" not in res["unpack_plan"] and res["unpack_plan"].count("tile W=1") == 3     # 3 bytes: no read-only pass
    res = _emulate_roundtrip(vector(19, 1, 128, BYTE), 1, stage=1)
    assert res["unpack_plan"].count("prefetch") == 1 and res["unpack_plan"].count("tile W=1") == 4
    # where it does not apply: rows of several words, other pitches, more row dimensions, too few rows unless forced
    for t in (vector(3000, 3, 512, BYTE), vector(3000, 4, 384, BYTE), vector(3000, 32, 512, BYTE), vector(3000, 4, 1024, BYTE),
              vector(3000, 8, 256, BYTE), vector(3000, 2, 128, BYTE), hvector(3, 1, 1 << 20, vector(1000, 4, 256, BYTE))):
        assert "prefetch" not in _emulate_roundtrip(t, 1, stage=1)["unpack_plan"], t
    assert "prefetch" not in _emulate_roundtrip(vector(5000, 1, 512, BYTE), 1)["unpack_plan"]
    assert "prefetch" not in _emulate_roundtrip(vector(5000, 1, 512, BYTE), 1, stage=0)["unpack_plan"]
    # left to itself the planner stages from 2^19 rows on (64 MiB of typed memory at 128-byte pitch)
    res = _emulate_roundtrip(vector(1 << 19, 1, 128, BYTE), 1)
    assert res["unpack_plan"].count("prefetch") == 1 and res["unpack_plan"].count("tile W=1 ux=1 ur=1 nt=6 ") == 4
    assert " grid=192" in res["unpack_plan"] and "prefetch bytes=524288 tile=1024 blocks=512 grid=512" in res["unpack_plan"]
    assert "prefetch" not in _emulate_roundtrip(vector((1 << 19) - 1, 1, 128, BYTE), 1)["unpack_plan"]
    # objects that abut fold into rows and are staged together; objects apart are an outer dimension
    res = _emulate_roundtrip(subarray((512, 512), (512, 4), (0, 0), "C", BYTE), 3, stage=1)
    assert "prefetch bytes=6144 " in res["unpack_plan"] and " rows=1536 " in res["unpack_plan"]
    # several row dimensions at 512-byte pitch: the outer dimensions are cut into chunks, each with its pass in front
    res = _emulate_roundtrip(hvector(5, 1, 1 << 20, vector(1000, 4, 512, BYTE)), 1, stage=1, stage_bytes=8192, typed_shift=2, position=1)
    lines = res["unpack_plan"].splitlines()
    assert len(lines) == 6 and lines[0] == "prefetch bytes=8000 tile=1024 blocks=8 grid=8", lines
    assert lines[1].startswith("tile W=4 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=2000 nrd=2 ") and lines[1].endswith(" grid=8"), lines
    assert lines[4] == "prefetch bytes=4000 tile=1024 blocks=4 grid=4" and " rows=1000 nrd=1 " in lines[5], lines
    assert res["unpack_prefetched_span"] == 20000
    res = _emulate_roundtrip(vector(512, 4, 512, BYTE), 3, stage=1)     # three objects apart: an outer dimension
    assert res["unpack_plan"].count("prefetch") == 1 and " rows=1536 nrd=2 " in res["unpack_plan"]


def test_emulated_ragged_runs_at_any_alignment():
    # run lengths that are no multiple of the word, odd strides, every relative misalignment of the
    # two sides: exact bytes, gaps untouched, duplicates only inside a run
    rng = random.Random(404)
    for run in (17, 31, 33, 64, 65, 66, 67, 100, 127, 255, 1023, 1030, 4049):
        for _ in range(3):
            stride = run + rng.choice((1, 3, 5, 7, 9, 62))
            rows = rng.randint(2, 9)
            res = _emulate_roundtrip(vector(rows, run, stride, BYTE), 1, typed_shift=rng.randint(0, 7),
                                     packed_shift=rng.randint(0, 7), position=rng.randint(0, 5))
            want_w = 16 if run > 32 else 4
            assert res["plan"].startswith(f"tile W={want_w} "), res["plan"]
            assert res["duplicates"] == rows * (-run % want_w)
    # 3D, ragged run, several tiles
    t = hvector(3, 1, 7 * 5003, hvector(7, 1, 5003, contiguous(4099, BYTE)))
    for ts in range(8):
        for ps in (0, 1, 2, 3, 5, 7):
            res = _emulate_roundtrip(t, 1, typed_shift=ts, packed_shift=ps, position=1)
            assert "W=16 ux=2 ur=2 " in res["plan"] and "n0=257 back=13 " in res["plan"]
    # 513 words: chunks of 256 pad the run least (768 slots against 1024)
    assert "W=8 ux=1 ur=4 nt=3 bx=256 n0=513 " in _emulate_roundtrip(t, 1, typed_shift=1, max_word=8)["plan"]
    assert "W=8 ux=1 ur=4 nt=3 bx=256 n0=513 back=5 " in _emulate_roundtrip(t, 1)["unpack_plan"]   # rows beyond 1 KiB
    res = _emulate_roundtrip(vector(5, 4100, 5000, BYTE), 1, max_word=4)
    assert "W=4 ux=1 ur=4 nt=3 bx=256 n0=1025 back=0 " in res["plan"]   # 1280 slots against 2048
    assert "W=16" in _emulate_roundtrip(contiguous(3000, BYTE), 1, typed_shift=1, packed_shift=1)["plan"]
    # run pieces (a run cut along its length): a last piece shorter than a word starts early and
    # overlaps the piece before it
    res = _emulate_roundtrip(vector(3, 1001, 1013, BYTE), 2, typed_shift=3, max_words_per_run=50)
    assert res["launches"] == 2 and "n0=50 back=0 " in res["plan"] and "n0=13 back=7 " in res["plan"]
    res = _emulate_roundtrip(vector(3, 803, 1013, BYTE), 2, max_words_per_run=50)   # 800 + 3: the 3 ride in a word
    assert res["launches"] == 2 and res["plan"].count("n0=1 back=0 ") == 1
    for run in range(16, 70):
        _emulate_roundtrip(vector(3, run, 80, BYTE), 2, max_words_per_run=1, typed_shift=run % 5)


def test_emulated_transposing_tiles():
    # short elements adjacent in the typed buffer along an outer dimension: tiles through LDS.
    # Ragged tile edges, every word width, elements of several words, outer dimensions, several
    # objects, a negative stride.
    def transposed(m, n, elem, esz, lead=None):
        """Column-major walk of a row-major m x n matrix of `elem` (leading dimension `lead` elements)."""
        lead = lead or n
        return hvector(n, 1, esz, vector(m, 1, lead, elem))
    for esz, w, words, tile in ((4, 4, 1, 64), (8, 8, 1, 64), (16, 16, 1, 32), (1, 1, 1, 128), (2, 2, 1, 128), (3, 1, 3, 77),
                                (12, 4, 3, 40), (24, 8, 3, 40), (32, 16, 2, 24), (20, 4, 5, 32), (28, 4, 7, 27), (48, 16, 3, 21), (64, 16, 4, 18)):
        elem = {4: FLOAT, 8: named("DOUBLE")}.get(esz, contiguous(esz, BYTE))
        for m, n in ((64, 64), (70, 33), (32, 200), (129, 65)):
            if m * n * esz > 300000:
                continue
            lead = max(n, -(-128 // esz))     # rows at least a memory line apart
            res = _emulate_roundtrip(transposed(m, n, elem, esz, lead), 1, typed_shift=3, packed_shift=1, position=2)
            ta, tb = min(tile, n), min(tile, m)
            if 2 * ta > tile and 2 * tb > tile:     # neither dimension thin: square tiles (cut at the matrix edge)
                assert res["plan"].startswith(f"xpose W={w} words={words} tile={ta}x{tb} a={n} b={m} outer=0 "), res["plan"]
            assert res["plan"].startswith(f"xpose W={w} words={words} tile="), res["plan"]
            assert res["unpack_plan"].startswith(f"xpose W={w} "), res["unpack_plan"]
            assert res["duplicates"] == 0
    # a padded leading dimension, three objects (the count becomes an outer dimension), and a batch of planes
    res = _emulate_roundtrip(transposed(40, 50, FLOAT, 4, lead=61), 3)
    assert res["plan"].startswith("xpose W=4 words=1 tile=50x40 a=50 b=40 outer=1 "), res["plan"]
    planes = hvector(3, 1, 40 * 61 * 4 + 12, transposed(40, 50, FLOAT, 4, lead=61))
    res = _emulate_roundtrip(planes, 2, typed_shift=1)
    assert res["plan"].startswith("xpose W=4 words=1 tile=50x40 a=50 b=40 outer=2 "), res["plan"]
    # an outer dimension nested between the two tiled ones
    t = hvector(48, 1, 8, hvector(2, 1, 48 * 8 * 40 + 64, vector(40, 1, 48, named("DOUBLE"))))
    res = _emulate_roundtrip(t, 1)
    assert res["plan"].startswith("xpose W=8 words=1 tile=48x40 a=48 b=40 outer=1 "), res["plan"]
    # rows walked backwards (negative stride along B)
    res = _emulate_roundtrip(hvector(36, 1, 4, hvector(45, 1, -36 * 4, FLOAT)), 1)
    assert res["plan"].startswith("xpose W=4 words=1 tile=36x45 a=36 b=45 "), res["plan"]
    # a narrower word forced: more words per element
    res = _emulate_roundtrip(transposed(64, 64, FLOAT, 4), 1, max_word=2)
    assert res["plan"].startswith("xpose W=2 words=2 tile=64x64 "), res["plan"]
    # thin matrices (records of a few fields turned into one array per field, and back): the short
    # dimension is covered whole and the tile grows along the other
    _chunks = lambda e: e // 256 * 256 if e > 256 else e     # noqa: E731  a grown edge is a whole number of 256-lane chunks
    rec = lambda f, n: hvector(f, 1, 8, vector(n, 1, f, named("DOUBLE")))      # noqa: E731  array of records -> field arrays
    fld = lambda f, n: hvector(n, 1, 8, vector(f, 1, n + 5, named("DOUBLE")))  # noqa: E731  field arrays -> array of records
    for f in (6, 8, 16, 31):
        res = _emulate_roundtrip(rec(f, 700), 1, typed_shift=1)
        assert res["plan"].startswith(f"xpose W=8 words=1 tile={f}x{_chunks(min(700, 1024, 6144 // (f | 1)))} a={f} b=700 "), res["plan"]
        res = _emulate_roundtrip(fld(f, 700), 2, packed_shift=3)
        assert res["plan"].startswith(f"xpose W=8 words=1 tile={_chunks(min(700, 1024, 6144 // f - 32))}x{f} a=700 b={f} outer=1 "), res["plan"]
    assert "xpose W=1 words=3 tile=7x" in _emulate_roundtrip(hvector(7, 1, 3, vector(900, 1, 7, contiguous(3, BYTE))), 1)["plan"]
    # records of three fields keep the row-by-row kernel for pack, of two fields for unpack too
    res = _emulate_roundtrip(rec(4, 700), 1)
    assert "xpose" in res["plan"] and "xpose" in res["unpack_plan"]
    res = _emulate_roundtrip(rec(3, 700), 1)
    assert "tile W" in res["plan"] and "xpose" in res["unpack_plan"]
    res = _emulate_roundtrip(rec(2, 700), 1)
    assert "tile W" in res["plan"] and "tile W" in res["unpack_plan"]
    # not applicable: too few elements, elements of too many words, B stride below two elements, or switched off
    assert "tile W" in _emulate_roundtrip(transposed(20, 40, FLOAT, 4), 1)["plan"]
    assert "tile W" in _emulate_roundtrip(transposed(64, 64, contiguous(31, BYTE), 31), 1)["plan"]     # 31 words of 1
    assert "tile W" in _emulate_roundtrip(transposed(64, 64, contiguous(80, BYTE), 80), 1)["plan"]
    assert "tile W" in _emulate_roundtrip(hvector(64, 1, 8, hvector(64, 1, 12, contiguous(8, BYTE))), 1)["plan"]   # overlapping rows
    res = _emulate_roundtrip(transposed(64, 64, FLOAT, 4), 1, allow_xpose=False)
    assert "tile W" in res["plan"]
    # rows of different outer index share memory lines here: L2 is left to merge them (no write-through)
    assert "tile W=1 ux=1 ur=4 nt=3 " in res["unpack_plan"], res["unpack_plan"]
    assert "ur=4 nt=3 " in _emulate_roundtrip(rec(2, 700), 1)["unpack_plan"]
    assert "tile W" in _emulate_roundtrip(transposed(64, 64, FLOAT, 4), 1, max_rows_per_launch=1000)["plan"]


def test_emulated_launch_splitting():
    t = hvector(7, 1, 4096, hvector(5, 1, 512, vector(9, 16, 32, BYTE)))
    one = _emulate_roundtrip(t, 3)
    assert one["launches"] == 1
    assert _emulate_roundtrip(t, 3, max_rows_per_launch=100)["launches"] > 1
    assert _emulate_roundtrip(t, 3, max_rows_per_launch=7)["launches"] > 10
    assert _emulate_roundtrip(t, 3, max_rows_per_launch=1)["launches"] == 3 * 7 * 5 * 9
    assert _emulate_roundtrip(t, 2, max_words_per_run=1, max_word=4)["launches"] == 4
    long_rows = vector(3, 5000, 6000, BYTE)
    assert _emulate_roundtrip(long_rows, 2, max_words_per_run=100, max_rows_per_launch=4)["launches"] > 4


def test_every_launch_fits_the_grid_limit():
    # The runtime launches no grid of 2^32 threads or more, i.e. at most 2^24 - 1 workgroups of 256.
    # Plans for row counts up to the 2^31 - 1 a call can name (planned at made-up addresses: nothing runs).
    limit = (1 << 24) - 1
    big = (1 << 31) - 1
    shapes = [
        (0, [1, big], [1, 512]),                    # one-byte rows: written through on unpack, one row per thread
        (0, [1, 1 << 30], [1, 16]),                 # rows that share lines
        (0, [3, (1 << 29) + 5], [1, 64]),
        (0, [4096, 1 << 27], [1, 8192]),            # 256 words per row: four rows per workgroup
        (0, [1 << 20, 1 << 12, 1 << 10], [1, 1 << 21, 1 << 34]),   # many x-chunks times many rows
        (0, [big], [1]),                            # one long run
        (0, [8, big, 2], [1, 16, 1 << 36]),
        (0, [8, 40000, 60000], [1, 8 * 60000, 8]),  # a matrix walked by columns: transposing tiles
    ]
    seen_capped = False
    for block in shapes:
        for unpack in (False, True):
            for batched in (False, True):
                launches = host_emul.plan_only(unpack, block, 1 << 50, 1, batched=batched)
                assert launches, block
                for l in launches:
                    assert 1 <= l["grid"] <= limit and l["grid"] * 256 < 1 << 32, (block, unpack, l)
                    assert l["grid"] <= l["tiles"] < 1 << 31
                    if l["kind"] in (1, 100):
                        assert l["grid"] == l["tiles"]      # these kernels take one tile per workgroup
                    seen_capped |= l["grid"] < l["tiles"] and l["kind"] == 0
                # the launches together cover every row once
                if all(l["kind"] == 0 for l in launches) and len(block[1]) == 2:
                    assert sum(l["rows"] for l in launches) == block[1][1]
    assert seen_capped


def test_override_keys_take_what_the_header_documents():
    # every key and value include/tp_pack.h lists is accepted, a few it does not list are refused,
    # and each key is put back to its default
    L = tp.lib()
    documented = {
        "word": ["0", "1", "2", "4", "8", "16"], "check_buffers": ["0", "1"], "nt": ["0", "1", "2", "3", "6", "7", "-1"],
        "ur": ["1", "4", "-1"], "xpose": ["0", "1"], "narrow_partial_rows": ["0", "1"], "unpack_rule": ["0", "1"],
        "stage": ["0", "1", "-1"], "stage_bytes": ["4096", str(1 << 30), str(16 << 20)], "stage_grid": ["256", "1", "0"], "grid": ["192", str(1 << 20), "0"],
        "max_rows_per_launch": ["1", "1000", str(1 << 30)], "max_words_per_run": ["1", "77", str(1 << 30)],
    }
    for key, values in documented.items():
        for v in values:   # the last value of each list is the default
            assert L.tp_set_override(key.encode(), v.encode()) == tp.TP_SUCCESS, (key, v)
    refused = {"word": ["3", "32", "-1"], "nt": ["4", "5", "8", "-2", "x", "", "3 "], "ur": ["0", "2", "8"], "xpose": ["2"],
               "stage": ["2", "-2"], "stage_bytes": ["4095", str((1 << 30) + 1)], "stage_grid": ["-1", str((1 << 20) + 1)], "grid": ["-1", str((1 << 20) + 1)],
               "unpack_rule": ["2"], "check_buffers": ["-1"], "narrow_partial_rows": ["7"],
               "max_rows_per_launch": ["0", str((1 << 30) + 1)], "max_words_per_run": ["0"], "nope": ["1"],
               "word ": ["4"]}
    for key, values in refused.items():
        for v in values:
            assert L.tp_set_override(key.encode(), v.encode()) == tp.TP_ERR_ARG, (key, v)
    assert L.tp_set_override(None, b"1") == tp.TP_ERR_ARG and L.tp_set_override(b"nt", None) == tp.TP_ERR_ARG


def test_emulated_objects_that_abut_are_merged():
    # extent == size: incount objects are one longer run / one longer stream
    assert "rows=1 " in _emulate_roundtrip(contiguous(64, BYTE), 5)["plan"]
    sub = subarray((8, 64), (8, 16), (0, 0), "C", BYTE)   # extent 512 = 8 rows of pitch 64
    assert "rows=40 nrd=1" in _emulate_roundtrip(sub, 5)["plan"]


def test_emulated_batch_of_different_types():
    # 71 requests of assorted types into one packed stream: batched launches of up to 40 requests,
    # plus the requests with too many row dimensions for a batch descriptor, which stay single launches
    rng = random.Random(77)
    types = _random_types(305, 69, allow_negative=False)
    types.insert(20, hvector(2, 1, 9000, hvector(3, 1, 1500, hvector(2, 1, 700, vector(3, 2, 100, hvector(2, 1, 40, INT16))))))
    types.insert(40, hvector(40, 1, 4, vector(33, 1, 40, FLOAT)))    # a transposing launch: stays single
    reqs, recipes = [], []
    typed_len = 0
    for t in types:
        h = tp.type_from_recipe(t)
        count = rng.randint(1, 2)
        disps = py.byte_displacements(t, count)
        span = max(disps) + 1
        origin = typed_len + rng.choice((0, 1, 2, 4, 8, 16))
        typed_len = origin + span + 16
        reqs.append({"block": tp.type_get_strided_block(h), "extent": tp.type_get_extent(h)[1], "count": count,
                     "origin": origin, "size": tp.type_size(h)})
        recipes.append((t, count, origin))
    total = sum(r["size"] * r["count"] for r in reqs)
    typed = W.random_bytes(5, typed_len)
    packed = np.full(total + 3, 0xEE, dtype=np.uint8)
    res = host_emul.transfer_batch(False, reqs, typed, packed, 3)
    assert (res["rc"], res["oob"], res["rewritten"]) == (0, 0, 0), res
    assert res["batches"] == 2 and 1 <= res["singles"] <= 30 and res["singles"] + 40 < len(types)
    expect = np.full(total + 3, 0xEE, dtype=np.uint8)
    pos = 3
    for t, count, origin in recipes:
        pos = cc.pack(typed, origin, count, t, expect, pos)
    assert pos == total + 3 and np.array_equal(packed, expect)
    assert (res["write_count"][3:] >= 1).all() and res["duplicates"] == int(res["write_count"].sum()) - total
    back = np.full(typed_len, 0xA5, dtype=np.uint8)
    res = host_emul.transfer_batch(True, reqs, back, packed, 3)
    assert (res["rc"], res["oob"]) == (0, 0), res
    # small requests keep plans that the batched kernel runs, also where a call of their own would write through
    assert res["batches"] == 2 and 1 <= res["singles"] <= 30
    if not any(py.has_overlap(t, count) for t, count, _ in recipes):
        assert res["rewritten"] == 0
    want = np.full(typed_len, 0xA5, dtype=np.uint8)
    pos = 3
    compared = 0
    for t, count, origin in recipes:
        if not py.has_overlap(t, count):
            pos = cc.unpack(expect, pos, want, origin, count, t)
            compared += 1
        else:
            pos += py.size(t) * count
    assert compared >= 50, compared   # of 71; overlapping maps (no unique unpack) stay the exception
    ok = np.ones(typed_len, dtype=bool)
    for t, count, origin in recipes:
        if py.has_overlap(t, count):
            ok[np.asarray(py.byte_displacements(t, count)) + origin] = False
    assert np.array_equal(back[ok], want[ok])


def test_batch_error_leaves_position_unchanged():
    L = tp.lib()
    t = tp.type_from_recipe(vector(3, 2, 4, BYTE))
    fake = 4096
    ptrs = (ctypes.c_void_p * 2)(fake, fake)
    cnts = (ctypes.c_int * 2)(1, 1)
    pos = ctypes.c_int64(2)
    bad = (ctypes.c_int32 * 2)(t, 999999)
    assert L.tp_pack_batch(2, ptrs, cnts, bad, fake, 100, ctypes.byref(pos), None) == tp.TP_ERR_TYPE
    good = (ctypes.c_int32 * 2)(t, t)
    assert L.tp_pack_batch(2, ptrs, cnts, good, fake, 13, ctypes.byref(pos), None) == tp.TP_ERR_TRUNCATE  # 2+6+6 > 13
    neg = (ctypes.c_int * 2)(1, -1)
    assert L.tp_unpack_batch(2, fake, 100, ctypes.byref(pos), ptrs, neg, good, None) == tp.TP_ERR_COUNT
    assert L.tp_pack_batch(-1, ptrs, cnts, good, fake, 100, ctypes.byref(pos), None) == tp.TP_ERR_ARG
    assert L.tp_pack_batch(2, None, cnts, good, fake, 100, ctypes.byref(pos), None) == tp.TP_ERR_ARG
    assert L.tp_pack_batch(0, None, None, None, None, 0, ctypes.byref(pos), None) == tp.TP_SUCCESS
    assert pos.value == 2


def test_multiply_shift_division_is_exact():
    # the kernels turn row indices into coordinates with this; checked against the hardware divide
    assert host_emul.fastdiv_mismatches(100000, 3000000, 12345) == 0


def test_handle_table_hammered_by_threads_in_the_host_build():
    # the library's type tree, handle table and commit, compiled for the host (tests/host_emul/types_emul.cpp):
    # eight threads build, commit, look up and free types at once, one node committed by all of them
    assert host_emul.types_hammer(8, 3000) == 0


def test_handle_table_and_commit_are_thread_safe():
    import threading

    recipe = W.configs.cfg5()["recipe"]
    shared = tp.type_from_recipe(recipe, commit=False)
    errors = []

    def worker(seed):
        try:
            rng = random.Random(seed)
            for _ in range(300):
                tp.type_commit(shared)                      # racing commits of one handle
                assert tp.type_get_strided_block(shared)[1] == [4096, 8, 16, 4]
                t = W.random_recipe(rng, rng.randint(1, 3))
                h = tp.type_from_recipe(t)
                assert tp.type_size(h) == cc.size(t)
                if h >= 12:
                    tp.type_free(h)
        except Exception as e:  # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(s,)) for s in range(8)]
    [t.start() for t in threads]
    [t.join() for t in threads]
    assert not errors, errors[:1]
    tp.type_free(shared)


def _deep_type(levels, run=3):
    """`levels` nested 2-element hvectors whose strides never let two levels merge."""
    t = contiguous(run, BYTE)
    stride = run + 1
    for _ in range(levels):
        t = hvector(2, 1, stride, t)
        stride = 2 * stride + 1
    return t


def test_many_dimensions():
    # 14 row dimensions plus the run: the looped (not unrolled) row decomposition, all 2^14 rows
    t = _deep_type(14)
    h = tp.type_from_recipe(t)
    start, counts, strides = tp.type_get_strided_block(h)
    assert counts == [3] + [2] * 14 and len(set(strides)) == 15
    res = _emulate_roundtrip(t, 1, typed_shift=1)
    assert "nrd=14" in res["plan"]
    # with two objects the count adds a 15th row dimension; 16 dimensions is the limit
    assert "nrd=15" in _emulate_roundtrip(_deep_type(14), 2)["plan"]
    assert tp.type_get_strided_block(tp.type_from_recipe(_deep_type(15)))[1] == [3] + [2] * 15
    assert "nrd=16" in _emulate_roundtrip(_deep_type(15), 2)["plan"]   # every row-dimension slot in use
    too_deep = tp.type_from_recipe(_deep_type(16), commit=False)
    with pytest.raises(tp.TpError) as e:
        tp.type_commit(too_deep)
    assert e.value.code == tp.TP_ERR_RANGE
    with pytest.raises(tp.TpError) as e:      # a type whose commit failed stays unusable
        tp.type_get_strided_block(too_deep)
    assert e.value.code == tp.TP_ERR_TYPE
