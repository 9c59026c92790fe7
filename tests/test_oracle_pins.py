"""Pins for the CPU oracle (both the Python interpreter and its C twin).

The oracle is the yardstick for the HIP library, so it is itself pinned to
things that are not the oracle: hand-enumerated type maps (tests/golden),
closed forms from the MPI definitions the paper restates in Sec. 2, numpy's own
slicing / as_strided as an independent reading of "subarray" and "strided",
the paper's lists of equivalent constructions (Sec. 2), and invariants.
"""
import os
import random

import numpy as np
import pytest
from numpy.lib.stride_tricks import as_strided

import workloads as W
from workloads import BYTE, DOUBLE, FLOAT, contiguous, hvector, named, subarray, vector
from oracle import typemap as py
from oracle import typemap_c as cc

INT16 = named("INT16")

TINY = {
    "vector_3_2_4_byte": vector(3, 2, 4, BYTE),
    "hvector_2_1_5_contig2": hvector(2, 1, 5, contiguous(2, BYTE)),
    "contig3_of_vector_2_1_2": contiguous(3, vector(2, 1, 2, BYTE)),
    "subarray_c_4x6": subarray((4, 6), (2, 3), (1, 2), "C", BYTE),
    "subarray_f_4x6": subarray((4, 6), (2, 3), (1, 2), "F", BYTE),
    "vector_2_1_2_float": vector(2, 1, 2, FLOAT),
    "vector_3_1_m2_byte": vector(3, 1, -2, BYTE),
    "hvector_2_2_7_int16": hvector(2, 2, 7, INT16),
    "vector_2_2_3_contig2_int16": vector(2, 2, 3, contiguous(2, INT16)),
    "subarray1d_of_vector": subarray((5,), (2,), (2,), "C", vector(2, 1, 2, BYTE)),
    "vector_0_2_4_byte": vector(0, 2, 4, BYTE),
    "subarray_empty_4x6": subarray((4, 6), (2, 0), (1, 2), "C", BYTE),
    "hvector_of_wide_subarray": hvector(3, 1, 32, subarray((6,), (4,), (0,), "C", INT16)),
    "vector_of_empty_subarray": vector(2, 1, 4, subarray((4, 6), (2, 0), (1, 2), "C", BYTE)),
}


def _read_golden(golden_dir):
    rows = {}
    with open(os.path.join(golden_dir, "tiny_type_maps.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, size, lb, ub, blocks = [c.strip() for c in line.split("|")]
            blk = [tuple(int(v) for v in b.split(":")) for b in blocks.split()]
            rows[name] = (int(size), int(lb), int(ub), blk)
    return rows


def test_golden_file_covers_every_tiny_recipe(golden_dir):
    assert set(_read_golden(golden_dir)) == set(TINY)


@pytest.mark.parametrize("name", sorted(TINY))
def test_tiny_type_maps_python(name, golden_dir):
    size, lb, ub, blocks = _read_golden(golden_dir)[name]
    t = TINY[name]
    assert list(py.type_map(t)) == blocks
    assert py.size(t) == size
    assert py.bounds(t) == (lb, ub)


@pytest.mark.parametrize("name", sorted(TINY))
def test_tiny_type_maps_c(name, golden_dir):
    size, lb, ub, blocks = _read_golden(golden_dir)[name]
    t = TINY[name]
    d, n = cc.blocks(t)
    assert list(zip(d.tolist(), n.tolist())) == blocks
    assert cc.measure(t) == (size, lb, ub)


# ------------------------------------------------------------ closed forms
@pytest.mark.parametrize("c,l,s,esz", [(5, 2, 3, "BYTE"), (7, 3, 3, "FLOAT"), (4, 1, 9, "DOUBLE"), (2, 4, 6, "INT16")])
def test_vector_closed_forms(c, l, s, esz):
    # for s >= l > 0: size = c*l*sizeof, extent = ((c-1)*s + l)*sizeof (MPI-3.1 Sec. 4.1.2)
    t = vector(c, l, s, named(esz))
    sz = py.NAMED_SIZE[esz]
    for o in (py, cc):
        assert o.size(t) == c * l * sz
        assert o.extent(t) == ((c - 1) * s + l) * sz


def test_config_sizes_closed_form():
    # packed sizes stated with the workloads: 512 B; 1 MiB; 2 MiB per object
    c1 = W.configs.cfg1()
    for r in c1["recipes"].values():
        assert py.size(r) == 512 and cc.size(r) == 512
    assert cc.extent(c1["recipes"]["vector"]) == 63 * 512 + 8
    for a0 in W.configs.A0_SWEEP:
        p = W.configs.cfg2_point(a0, 1 << 20)
        assert cc.size(p["recipe"]) == 1 << 20 == p["packed_bytes"]
    c5 = W.configs.cfg5()
    assert cc.size(c5["recipe"]) == 2 * 1024 * 1024
    # 26 halo regions of the 506^3 interior with width 3: 6 faces, 12 edges, 8 corners
    c3 = W.configs.cfg3()
    total = sum(cc.size(r) for r in c3["send"])
    assert total == 8 * (6 * 3 * 506 * 506 + 12 * 3 * 3 * 506 + 8 * 27) == 37308096
    assert all(cc.extent(r) == 8 * 512 ** 3 for r in c3["send"])


# --------------------------------------------- numpy as an independent reading
@pytest.mark.parametrize("order", ["C", "F"])
@pytest.mark.parametrize("oracle", [py, cc], ids=["py", "c"])
def test_subarray_equals_numpy_slicing(order, oracle):
    # a C-order subarray of a row-major array is numpy's basic slice of it; Fortran order is
    # the same slice of the column-major view (sizes deliberately all different)
    sizes, subs, starts = (5, 7, 6), (2, 4, 3), (1, 2, 3)
    raw = W.random_bytes(11, int(np.prod(sizes)) * 4)
    a = raw.view(np.float32).reshape(sizes, order=order)
    sel = a[tuple(slice(s, s + n) for s, n in zip(starts, subs))]
    expect = np.frombuffer(sel.tobytes(order=order), dtype=np.uint8)
    t = subarray(sizes, subs, starts, order, FLOAT)
    out = np.zeros(expect.size, dtype=np.uint8)
    assert oracle.pack(raw, 0, 1, t, out, 0) == expect.size
    assert np.array_equal(out, expect)


@pytest.mark.parametrize("oracle", [py, cc], ids=["py", "c"])
def test_vector_equals_numpy_reshape(oracle):
    count, bl, stride = 9, 3, 5
    raw = W.random_bytes(12, count * stride * 2)
    a = raw.view(np.int16).reshape(count, stride)
    expect = np.ascontiguousarray(a[:, :bl]).view(np.uint8).reshape(-1)
    out = np.zeros(expect.size, dtype=np.uint8)
    oracle.pack(raw, 0, 1, vector(count, bl, stride, INT16), out, 0)
    assert np.array_equal(out, expect)


@pytest.mark.parametrize("oracle", [py, cc], ids=["py", "c"])
def test_nested_hvector_equals_as_strided(oracle):
    # hvector(c2, l2, sb2, hvector(c1, l1, sb1, INT16)) read with numpy's strided view:
    # shape (c2, l2, c1, l1), byte strides (sb2, extent(inner), sb1, 2);
    # extent(inner) = (c1-1)*sb1 + l1*2 for sb1 >= l1*2 (closed form, written here by hand)
    c1, l1, sb1 = 3, 2, 10
    c2, l2, sb2 = 4, 2, 100
    ext_inner = (c1 - 1) * sb1 + l1 * 2
    raw = W.random_bytes(13, 1024)
    view = as_strided(raw.view(np.int16), shape=(c2, l2, c1, l1), strides=(sb2, ext_inner, sb1, 2))
    expect = np.ascontiguousarray(view).view(np.uint8).reshape(-1)
    t = hvector(c2, l2, sb2, hvector(c1, l1, sb1, INT16))
    out = np.zeros(expect.size, dtype=np.uint8)
    assert oracle.pack(raw, 0, 1, t, out, 0) == expect.size
    assert np.array_equal(out, expect)
    assert oracle.extent(t) == (c2 - 1) * sb2 + (l2 - 1) * ext_inner + ext_inner


def test_halo_regions_equal_numpy_slices_small_grid():
    # the 26 send regions of a 12^3 float64 grid, ghost width 2, against numpy slices
    n, r = 12, 2
    c3 = W.configs.cfg3(n, r)
    grid = W.random_grid_f64(c3["seed"], c3["grid_shape"])
    raw = grid.reshape(-1).view(np.uint8)
    for rec, reg in zip(c3["send"], c3["send_region"]):
        sel = grid[tuple(slice(a, b) for a, b in reg)]
        expect = np.ascontiguousarray(sel).reshape(-1).view(np.uint8)
        out = np.zeros(expect.size, dtype=np.uint8)
        cc.pack(raw, 0, 1, rec, out, 0)
        assert np.array_equal(out, expect)


def test_cfg4_full_size_equals_numpy_reshape():
    # 2^24 runs of 3 bytes at 64-byte stride, source offset 5: full size through the C oracle
    p = W.configs.cfg4_point(3)
    raw = W.fills.counter_bytes_numpy(p["seed"], 0, p["source_bytes"])
    k = 5
    expect = np.ascontiguousarray(raw[k:k + W.configs.CFG4_COUNT * 64].reshape(-1, 64)[:, :3]).reshape(-1)
    out = np.zeros(p["packed_bytes"], dtype=np.uint8)
    assert cc.pack(raw, k, 1, p["recipe"], out, 0) == p["packed_bytes"]
    assert np.array_equal(out, expect)
    out2 = np.zeros_like(out)
    cc.pack(raw, 0, 1, p["recipe_subarray"](k), out2, 0, nthreads=4)
    assert np.array_equal(out2, expect)


# ---------------------------------------- the paper's equivalent constructions
def _rows(e0, a0):
    """Seven constructions of one row of e0 floats in an a0-float-wide array (paper Sec. 2)."""
    return [
        contiguous(e0, FLOAT),
        contiguous(e0 * 4, BYTE),
        vector(1, e0, 1, FLOAT),
        vector(e0, 4, 4, BYTE),
        hvector(e0 * 4, 1, 1, BYTE),
        subarray((a0,), (e0,), (0,), "C", FLOAT),
        subarray((a0 * 4,), (e0 * 4,), (0,), "C", BYTE),
    ]


def _planes(e0, e1, a0, a1):
    """Constructions of a plane of e1 rows (paper Sec. 2); a0 counts floats per allocation row."""
    out = [
        vector(e1, e0, a0, FLOAT),
        vector(e1, e0 * 4, a0 * 4, BYTE),
        subarray((a1, a0), (e1, e0), (0, 0), "C", FLOAT),
        subarray((a1, a0 * 4), (e1, e0 * 4), (0, 0), "C", BYTE),
    ]
    out += [hvector(e1, 1, a0 * 4, row) for row in _rows(e0, a0)]
    # for the subarray rows (extent = one allocation row) stride-1 vectors and a 1D subarray also work
    for row in _rows(e0, a0)[5:]:
        out.append(vector(e1, 1, 1, row))
        out.append(subarray((a1,), (e1,), (0,), "C", row))
    return out


def _cuboids(e, a):
    e0, e1, e2 = e
    a0, a1, a2 = a
    out = [hvector(e2, 1, a0 * 4 * a1, p) for p in _planes(e0, e1, a0, a1)]
    out.append(subarray((a2, a1, a0), (e2, e1, e0), (0, 0, 0), "C", FLOAT))
    out.append(subarray((a2, a1, a0 * 4), (e2, e1, e0 * 4), (0, 0, 0), "C", BYTE))
    return out


def test_paper_equivalent_constructions_pack_identically():
    e, a = (5, 3, 4), (8, 6, 5)
    raw = W.random_bytes(14, a[0] * 4 * a[1] * a[2])
    arr = raw.view(np.float32).reshape(a[2], a[1], a[0])
    expect = np.ascontiguousarray(arr[:e[2], :e[1], :e[0]]).reshape(-1).view(np.uint8)
    for t in _cuboids(e, a):
        out = np.zeros(expect.size, dtype=np.uint8)
        assert cc.pack(raw, 0, 1, t, out, 0) == expect.size, t
        assert np.array_equal(out, expect), t
        assert py.byte_displacements(t) == py.byte_displacements(_cuboids(e, a)[0])


def test_row_constructions_differ_in_extent_only():
    rows = _rows(5, 8)
    maps = {tuple(py.byte_displacements(t)) for t in rows}
    assert len(maps) == 1
    assert {py.extent(t) for t in rows} == {20, 32}   # subarray rows span the allocation row


# ------------------------------------------------------------------ invariants
def _random_types(seed, n, **kw):
    rng = random.Random(seed)
    out = []
    while len(out) < n:
        t = W.random_recipe(rng, rng.randint(1, 4), **kw)
        if py.size(t) <= 4096:
            out.append(t)
    return out


def test_c_twin_equals_python_on_random_trees():
    for t in _random_types(101, 400, allow_negative=True, allow_zero=True, allow_overlap=True):
        d, n = cc.blocks(t, 2)
        ex = py.extent(t)
        expect = [b for obj in range(2) for b in py.type_map(t, obj * ex)]
        assert list(zip(d.tolist(), n.tolist())) == expect, t
        assert cc.measure(t) == (py.size(t), *py.bounds(t)), t


def test_pack_unpack_roundtrip_and_poison():
    rng = random.Random(7)
    for t in _random_types(102, 150, allow_negative=True):
        incount = rng.randint(1, 3)
        if py.has_overlap(t, incount):
            continue
        lb, ub = py.bounds(t)
        ex = ub - lb
        lo = min(0, lb, lb + (incount - 1) * ex)
        hi = max(0, ub, ub + (incount - 1) * ex)
        origin = -lo + 3
        n = hi - lo + 9
        src = W.random_bytes(rng.randrange(1 << 30), n)
        size = py.size(t) * incount
        for o in (py, cc):
            packed = np.full(size + 5, 0xEE, dtype=np.uint8)
            assert o.pack(src, origin, incount, t, packed, 2) == 2 + size
            assert packed[0] == packed[1] == 0xEE and (packed[2 + size:] == 0xEE).all()
            dst = np.full(n, 0xA5, dtype=np.uint8)
            assert o.unpack(packed, 2, dst, origin, incount, t) == 2 + size
            sel = np.asarray(py.byte_displacements(t, incount), dtype=np.int64) + origin
            mask = np.zeros(n, dtype=bool)
            mask[sel] = True
            assert np.array_equal(dst[mask], src[mask])
            assert (dst[~mask] == 0xA5).all()
            # incount objects == incount single packs at origin + i*extent
            one = np.zeros(size, dtype=np.uint8)
            p = 0
            for i in range(incount):
                p = o.pack(src, origin + i * ex, 1, t, one, p)
            assert np.array_equal(one, packed[2:2 + size])


def test_same_byte_set_in_other_order_packs_differently():
    # columns-of-rows vs rows-of-columns select the same bytes but in another order
    a = hvector(3, 1, 8, hvector(2, 1, 2, BYTE))     # 0,2, 8,10, 16,18
    b = hvector(2, 1, 2, hvector(3, 1, 8, BYTE))     # 0,8,16, 2,10,18
    assert sorted(py.byte_displacements(a)) == sorted(py.byte_displacements(b))
    assert py.byte_displacements(a) != py.byte_displacements(b)
    raw = np.arange(32, dtype=np.uint8)
    oa, ob = np.zeros(6, np.uint8), np.zeros(6, np.uint8)
    cc.pack(raw, 0, 1, a, oa, 0), cc.pack(raw, 0, 1, b, ob, 0)
    assert oa.tolist() == [0, 2, 8, 10, 16, 18] and ob.tolist() == [0, 8, 16, 2, 10, 18]


def test_threaded_c_oracle_equals_single_thread():
    t = W.configs.cfg5()["recipe"]
    ex = cc.extent(t)
    src = W.random_bytes(5, ex * 3)
    a = np.zeros(cc.size(t) * 3, np.uint8)
    b = np.zeros_like(a)
    cc.pack(src, 0, 3, t, a, 0, nthreads=1)
    cc.pack(src, 0, 3, t, b, 0, nthreads=7)
    assert np.array_equal(a, b)
    t2 = W.configs.cfg2_point(16, 1 << 20)["recipe"]
    src = W.random_bytes(6, 512 * 512 * 512)
    a = np.zeros(1 << 20, np.uint8)
    b = np.zeros_like(a)
    cc.pack(src, 0, 1, t2, a, 0, nthreads=1)
    cc.pack(src, 0, 1, t2, b, 0, nthreads=5)
    assert np.array_equal(a, b)
    back = np.zeros_like(src)
    cc.unpack(b, 0, back, 0, 1, t2, nthreads=3)
    sel = src.reshape(512, 512, 512)[:256, :256, :16]
    assert np.array_equal(back.reshape(512, 512, 512)[:256, :256, :16], sel)
    assert int(back.sum(dtype=np.int64)) == int(sel.sum(dtype=np.int64))


def test_truncation_and_bounds_are_errors():
    t = vector(3, 2, 4, BYTE)
    src = np.zeros(10, np.uint8)
    for o in (py, cc):
        with pytest.raises(ValueError):
            o.pack(src, 0, 1, t, np.zeros(5, np.uint8), 0)
        with pytest.raises(IndexError):
            o.pack(src[:9], 0, 1, t, np.zeros(6, np.uint8), 0)


# --------------------------------------------------------------- has_overlap
def test_has_overlap_on_hand_worked_cases():
    """`has_overlap` decides whether a test may compare an unpack at all, so it is pinned in both
    directions by cases worked out by hand (none of them computed with the oracle)."""
    # two blocks of two bytes one byte apart: bytes 0 1 | 1 2
    assert py.has_overlap(vector(2, 2, 1, BYTE))
    # a stride of zero puts both copies on the same byte
    assert py.has_overlap(hvector(2, 1, 0, BYTE))
    # 4-byte elements placed 2 bytes apart
    assert py.has_overlap(hvector(3, 1, 2, FLOAT))
    # a negative stride that walks back over the first block: bytes 0..3 then -2..1
    assert py.has_overlap(hvector(2, 1, -2, contiguous(4, BYTE)))
    # the nested workload: rows 16384 apart inside planes 8192 apart, (j, i) = (1, 0) and (0, 2) collide
    assert py.has_overlap(W.configs.cfg5()["recipe"])
    # disjoint: blocks that touch but do not cross, gaps, negative strides that clear the block
    assert not py.has_overlap(vector(3, 2, 4, BYTE))
    assert not py.has_overlap(vector(2, 2, 2, BYTE))            # bytes 0 1 | 2 3: adjacent
    assert not py.has_overlap(hvector(2, 1, -4, contiguous(4, BYTE)))
    assert not py.has_overlap(contiguous(2, vector(2, 1, 2, BYTE)))   # extent 3: bytes 0 2 | 3 5
    assert not py.has_overlap(W.configs.cfg1()["recipes"]["vector"])
    assert not py.has_overlap(W.configs.cfg2_point(4, 1 << 12)["recipe"])
    assert not py.has_overlap(subarray((4, 6), (2, 3), (1, 2), "C", BYTE))
    # several objects sit one extent apart, and the extent spans every copy: objects of a disjoint
    # type never collide, objects of a colliding type still do
    assert not py.has_overlap(vector(3, 2, 4, BYTE), 3)
    assert not py.has_overlap(hvector(2, 1, -4, contiguous(4, BYTE)), 2)
    assert py.has_overlap(vector(2, 2, 1, BYTE), 2)


def test_has_overlap_equals_a_byte_census_on_random_trees():
    # brute force, another way round: mark every selected byte in an array and look for a second mark
    both = {True: 0, False: 0}
    for t in _random_types(909, 400, allow_negative=True):
        incount = 2
        blocks = [b for obj in range(incount) for b in py.type_map(t, obj * py.extent(t))]
        if not blocks:
            assert not py.has_overlap(t, incount)
            continue
        lo = min(d for d, _ in blocks)
        marks = np.zeros(max(d + n for d, n in blocks) - lo, dtype=np.int32)
        for d, n in blocks:
            marks[d - lo:d - lo + n] += 1
        expect = bool((marks > 1).any())
        assert py.has_overlap(t, incount) == expect, t
        both[expect] += 1
    assert both[True] >= 20 and both[False] >= 100, both
