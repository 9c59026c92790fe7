"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle,
byte for byte, on the same seeded inputs.  Needs a real MI355X (-m gpu)."""
import os
import random
import sys

import numpy as np
import pytest

import workloads as W
from workloads import BYTE, DOUBLE, FLOAT, contiguous, hvector, named, subarray, vector
from oracle import typemap as py
from oracle import typemap_c as cc
from paper_2012_14363_amd import binding as tp

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    tp.lib()  # fails loudly if the HIP library is not built
    return torch.device("cuda:0")


def to_dev(a: np.ndarray, dev):
    return torch.from_numpy(a).to(dev)


def roundtrip(t, incount, dev, *, typed_shift=0, packed_shift=0, position=0, seed=0, check_unpack=True,
              pinned_packed=False):
    """pack on the GPU == oracle pack; unpack on the GPU into a poisoned buffer == oracle unpack."""
    h = tp.type_from_recipe(t)
    size = tp.type_size(h) * incount
    ex = tp.type_get_extent(h)[1]
    d, n = cc.blocks(t, incount)
    lo = min(0, int(d.min())) if d.size else 0
    hi = max(0, int((d + n).max())) if d.size else 0
    pad = 64
    origin = -lo + pad + typed_shift
    nbytes = hi - lo + 2 * pad + typed_shift
    typed_h = W.random_bytes(seed, nbytes)
    typed_d = to_dev(typed_h, dev)
    if pinned_packed:
        store = torch.full((position + size + 64,), 0xEE, dtype=torch.uint8).pin_memory()
    else:
        store = torch.full((position + size + 64,), 0xEE, dtype=torch.uint8, device=dev)
    packed_d = store[packed_shift:packed_shift + position + size]
    new_pos = tp.pack(typed_d.data_ptr() + origin, incount, h, packed_d, position + size, position)
    assert new_pos == position + size
    plans = {"pack": tp.last_plan(), "unpack": ""}
    expect = np.full(position + size, 0xEE, dtype=np.uint8)
    cc.pack(typed_h, origin, incount, t, expect, position)
    got = store.cpu().numpy()
    assert np.array_equal(got[packed_shift:packed_shift + position + size], expect), (t, tp.last_plan())
    assert (got[:packed_shift] == 0xEE).all() and (got[packed_shift + position + size:] == 0xEE).all()

    if check_unpack and not pinned_packed:
        dst_d = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device=dev)
        new_pos = tp.unpack(packed_d, position + size, position, dst_d.data_ptr() + origin, incount, h)
        assert new_pos == position + size
        want = np.full(nbytes, 0xA5, dtype=np.uint8)
        cc.unpack(expect, position, want, origin, incount, t)
        plans["unpack"] = tp.last_plan()
        assert np.array_equal(dst_d.cpu().numpy(), want), (t, tp.last_plan())
    if h >= 12:
        tp.type_free(h)
    return plans


# ------------------------------------------------------------------ small and ragged
def test_random_small_types(dev):
    rng = random.Random(401)
    done = compared = 0
    while done < 120:
        t = W.random_recipe(rng, rng.randint(1, 4), allow_negative=True)
        if py.size(t) > 4096:
            continue
        incount = rng.randint(1, 3)
        overlap = py.has_overlap(t, incount)
        say("random type", done, t, "incount", incount)
        roundtrip(t, incount, dev, typed_shift=rng.choice((0, 1, 2, 4, 8)), packed_shift=rng.choice((0, 1, 2, 4, 8)),
                  position=rng.choice((0, 3, 16)), seed=done, check_unpack=not overlap)
        done += 1
        compared += not overlap
    # a type whose map overlaps itself has no unique unpack and is only packed; that must stay the exception
    assert compared >= 90, compared


def _medium_recipe(rng):
    """A non-overlapping nested type of up to a few MiB: a run of 1..6000 bytes (BYTE, INT16, FLOAT or
    DOUBLE elements) under 1-3 levels of vector / hvector / subarray whose strides clear the child's extent."""
    elem = rng.choice(("BYTE", "BYTE", "INT16", "FLOAT", "DOUBLE"))
    esz = py.NAMED_SIZE[elem]
    run_elems = max(1, rng.choice((1, 2, 3, 5, 8, 24, 61, 64, 100, 257, 1000, 6000)) // esz)
    t = contiguous(run_elems, named(elem))
    ext = run_elems * esz
    budget = 4 << 20
    for _ in range(rng.randint(1, 3)):
        count = rng.choice((1, 2, 3, 7, 16, 33, 64, 200))
        count = max(1, min(count, budget // max(1, cc.size(t))))
        kind = rng.choice(("hvector", "vector", "subarray"))
        if kind == "hvector":
            stride = ext + rng.choice((0, 1, 3, 8, 16, 100, 4096))
            t = hvector(count, 1, stride, t)
        elif kind == "vector":
            bl = rng.choice((1, 2, 3))
            t = vector(count, bl, bl + rng.choice((0, 1, 2, 5)), t)
        else:
            size = count + rng.choice((0, 1, 5))
            t = subarray((size, 3), (count, rng.choice((1, 2, 3))), (rng.randint(0, size - count), 0),
                         rng.choice(("C", "F")), t)
        ext = cc.extent(t)
        budget = max(1, budget)
    return t


def test_random_medium_types(dev):
    # seeded fuzz over shapes far larger than the CPU emulation can afford: every kernel variant,
    # odd alignments, several objects, pack and unpack, against the C oracle
    rng = random.Random(777)
    kinds = set()
    for i in range(150):
        t = _medium_recipe(rng)
        incount = rng.choice((1, 1, 2, 3))
        if cc.size(t) * incount > (8 << 20) or cc.extent(t) * incount > (256 << 20):
            continue
        say("medium type", i, "size", cc.size(t), "extent", cc.extent(t), "incount", incount)
        plans = roundtrip(t, incount, dev, typed_shift=rng.choice((0, 0, 1, 2, 3, 4, 8, 16)),
                          packed_shift=rng.choice((0, 0, 1, 2, 3, 4, 8)), position=rng.choice((0, 0, 1, 5, 16)), seed=i)
        kinds.update(line.split(" ux=")[0] for line in (plans["pack"] + plans["unpack"]).splitlines())
    say("variants seen:", sorted(kinds))
    assert {"tile W=1", "tile W=4", "tile W=16"} <= kinds


def test_fewer_workgroups_than_tiles(dev):
    # a launch of more tiles than a grid may have workgroups runs on fewer workgroups, each taking every
    # gridDim-th tile; forced here with a handful of workgroups on launches of hundreds of tiles
    try:
        for grid in (1, 7, 64):
            tp.set_override("grid", grid)
            for t, incount in ((vector(20011, 3, 64, BYTE), 1), (vector(3001, 200, 512, BYTE), 2),
                               (hvector(5, 1, 37 * 20480, hvector(37, 1, 20480, contiguous(4100, BYTE))), 1),
                               (contiguous(3 << 20, BYTE), 1)):
                say("grid", grid, "type", t[0], t[1])
                plans = roundtrip(t, incount, dev, typed_shift=3, packed_shift=1, position=5, seed=grid)
                assert f" grid={grid}" in plans["pack"] and f" grid={grid}" in plans["unpack"], plans
    finally:
        tp.set_override("grid", 0)


@pytest.mark.parametrize("a0", [1, 2, 3, 4, 8, 16, 24, 48, 64, 200, 512, 1040, 4048, 4100, 4112, 20000])
def test_tile_shapes_and_ragged_tails(dev, a0):
    say("tile shapes a0", a0)
    # several tiles in every direction plus a ragged tail, 3D with incount and 2D
    roundtrip(hvector(5, 1, 37 * 20480, hvector(37, 1, 20480, contiguous(a0, BYTE))), 2, dev, seed=a0)
    roundtrip(vector(1031, a0, a0 + 16, BYTE), 1, dev, seed=a0 + 1)


@pytest.mark.parametrize("run", [17, 33, 64, 67, 127, 1030, 4049, 70001])
def test_ragged_runs_at_any_alignment(dev, run):
    # runs at odd addresses and of odd lengths move in 16-byte words all the same (unaligned
    # accesses, last word pulled back); every relative misalignment of the two sides, exact
    # writes (poisoned gaps), 2D and 3D
    say("ragged runs, run", run)
    rng = random.Random(run)
    want = "tile W=16 " if run > 32 else "tile W=4 "
    for ts in (0, 1, 2, 3, 7, 13):
        for ps in (0, 1, 2, 3, 6, 15):
            pitch = run + rng.choice((1, 3, 5, 61))
            plans = roundtrip(vector(41, run, pitch, BYTE), rng.randint(1, 2), dev,
                              typed_shift=ts, packed_shift=ps, position=rng.randint(0, 3), seed=run + ts)
            # rows that are not whole aligned 128-byte lines and closer together than a page are
            # written through, one row per thread, in words of an eighth of the row at most; rows
            # further apart in 4-byte words, or 8-byte words beyond 1 KiB
            if pitch < 4096:
                narrow = f"tile W={min(16, 1 << ((run // 8).bit_length() - 1))} ux=1 ur=1 nt=7 "
            else:
                narrow = "tile W=4 " if run <= 1024 else "tile W=8 "
            assert plans["pack"].startswith(want) and plans["unpack"].startswith(narrow), plans
    plans = roundtrip(hvector(3, 1, 9 * (run + 7), hvector(9, 1, run + 7, contiguous(run, BYTE))), 2, dev,
                      typed_shift=3, packed_shift=1, seed=run)
    assert want in plans["pack"]
    try:   # and byte-wide words give the same bytes
        tp.set_override("word", 1)
        plans = roundtrip(vector(41, run, run + 3, BYTE), 1, dev, typed_shift=1, seed=run)
        assert "tile W=1 " in plans["pack"] and "tile W=1 " in plans["unpack"]
    finally:
        tp.set_override("word", 0)


def dev_base_mod_512(dev):
    return torch.empty(1 << 20, dtype=torch.uint8, device=dev).data_ptr() % 512


def test_staged_unpack_of_tiny_rows(dev):
    # a million rows or more of one word each at 512-, 256- or 128-byte pitch: per 16 MiB of packed bytes a
    # read-only pass and store passes over rows 512 bytes apart; exact bytes, gaps untouched, any addresses
    for run, pitch, rows, ts, ps, pos in ((1, 512, (1 << 20) + 77, 0, 0, 0), (2, 512, (1 << 20) + 3, 1, 3, 5),
                                          (16, 512, (1 << 21) + 1, 8, 0, 0), (4, 256, (5 << 20) + 333, 2, 1, 1),
                                          (1, 128, (17 << 20) + 9, 0, 5, 2)):
        say("staged unpack, run", run, "pitch", pitch, "rows", rows)
        plans = roundtrip(vector(rows, run, pitch, BYTE), 1, dev, typed_shift=ts, packed_shift=ps, position=pos, seed=rows)
        passes = 512 // pitch
        chunks = -(-rows * run // (16 << 20))
        assert plans["unpack"].count("prefetch") == chunks, plans["unpack"]
        assert plans["unpack"].count(f"tile W={run} ux=1 ur=1 nt=6 ") == chunks * passes, plans["unpack"]
        assert "prefetch" not in plans["pack"]
    # rows in the last line of their 512-byte block are left unstaged (no gain there); torch aligns its blocks to 512
    plans = roundtrip(vector((1 << 20) + 5, 8, 512, BYTE), 1, dev, typed_shift=330, seed=8)
    assert (dev_base_mod_512(dev) + 64 + 330) % 512 >= 384 and "prefetch" not in plans["unpack"] and "nt=7" in plans["unpack"]
    # three row dimensions at 512-byte pitch, two objects apart
    say("staged unpack, 3D")
    plans = roundtrip(hvector(40, 1, 300 * 512 + 64, vector(300, 8, 512, BYTE)), 90, dev, typed_shift=4, position=3, seed=9)
    assert plans["unpack"].count("prefetch") == 1 and " nrd=3 " in plans["unpack"] and " grid=192" in plans["unpack"], plans["unpack"]
    try:   # forced on a short message, with small chunks and few workgroups; and switched off
        tp.set_override("stage", 1)
        tp.set_override("stage_bytes", 8192)
        tp.set_override("stage_grid", 8)
        plans = roundtrip(vector(70001, 2, 256, BYTE), 1, dev, typed_shift=1, seed=5)
        assert plans["unpack"].count("prefetch") == 18 and " grid=8" in plans["unpack"], plans["unpack"][:300]
        tp.set_override("stage", 0)
        plans = roundtrip(vector((1 << 20) + 77, 1, 512, BYTE), 1, dev, seed=6)
        assert "prefetch" not in plans["unpack"] and "nt=7" in plans["unpack"]
    finally:
        tp.set_override("stage", -1)
        tp.set_override("stage_bytes", 16 << 20)
        tp.set_override("stage_grid", 0)


def test_transposing_tiles(dev):
    # short elements adjacent along an outer dimension (a matrix walked column by column): tiles
    # through LDS, both directions, ragged edges, every word width, elements of several words,
    # outer dimensions, odd addresses
    def transposed(m, n, elem, esz, lead=None):
        return hvector(n, 1, esz, vector(m, 1, lead or n, elem))
    for esz, w in ((4, 4), (8, 8), (16, 16), (1, 1), (2, 2), (3, 1), (12, 4), (20, 4), (24, 8), (32, 16), (48, 16), (64, 16)):
        elem = {4: FLOAT, 8: DOUBLE}.get(esz, contiguous(esz, BYTE))
        for m, n, lead in ((64, 64, 128), (70, 133, 150), (257, 130, 131), (1000, 384, None), (33, 2049, 2050)):
            if m * n * esz > (12 << 20):
                continue
            say("transposing tiles", esz, m, n, lead)
            plans = roundtrip(transposed(m, n, elem, esz, lead), 1, dev, typed_shift=esz * 3 + 1, packed_shift=1,
                              position=5, seed=m + n)
            assert plans["pack"].startswith(f"xpose W={w} words={esz // w} ") and f" a={n} b={m} " in plans["pack"], plans
            assert plans["unpack"].startswith("xpose"), plans
    plans = roundtrip(hvector(3, 1, 300 * 200 * 8 + 24, transposed(300, 200, DOUBLE, 8)), 2, dev, typed_shift=1, seed=7)
    assert plans["pack"].startswith("xpose W=8 words=1 tile=64x64 a=200 b=300 outer=2 "), plans
    plans = roundtrip(hvector(100, 1, 4, hvector(90, 1, -100 * 4, FLOAT)), 3, dev, seed=8)
    assert plans["pack"].startswith("xpose W=4 words=1 tile=64x64 a=100 b=90 outer=1 "), plans
    # thin matrices: an array of records turned into one array per field, and back
    for f in (3, 4, 8, 16, 31):
        say("thin transposes, fields", f)
        plans = roundtrip(hvector(f, 1, 8, vector(100003, 1, f, DOUBLE)), 1, dev, typed_shift=1, packed_shift=3, seed=f)
        assert plans["unpack"].startswith(f"xpose W=8 words=1 tile={f}x{max(256, min(1024, 6144 // (f | 1)) // 256 * 256) if f < 31 else 198} "), plans
        assert plans["pack"].startswith("xpose" if f >= 4 else "tile W"), plans
        plans = roundtrip(hvector(50021, 1, 4, vector(f, 1, 50021 + 7, FLOAT)), 2, dev, typed_shift=4, position=1, seed=f)
        assert plans["unpack"].startswith("xpose W=4 words=1 tile=") and f"x{f} a=50021 b={f} outer=1 " in plans["unpack"], plans
    # the same bytes with the kernel switched off
    try:
        tp.set_override("xpose", 0)
        plans = roundtrip(transposed(257, 130, DOUBLE, 8, 131), 1, dev, seed=9)
        assert plans["pack"].startswith("tile W=2 ")
    finally:
        tp.set_override("xpose", 1)


def test_transposed_matrix_full_size(dev):
    # 4096 x 4096 float64 walked column by column: the packed stream is the transposed matrix
    # (numpy's transpose is the reference, the C oracle agrees on the leading part), and unpacking it
    # restores the matrix
    n = 4096
    say("full-size transpose: generating")
    a_h = W.random_grid_f64(4242, (n, n))
    a = to_dev(a_h.reshape(-1).view(np.uint8), dev)
    t = hvector(n, 1, 8, vector(n, 1, n, DOUBLE))
    h = tp.type_from_recipe(t)
    size = tp.type_size(h)
    assert size == n * n * 8 and tp.type_get_strided_block(h) == (0, [8, n, n], [1, 8 * n, 8])
    out = torch.zeros(size + 8, dtype=torch.uint8, device=dev)
    say("full-size transpose: pack")
    assert tp.pack(a, 1, h, out, size + 8, 8) == size + 8
    assert tp.last_plan().startswith("xpose W=8 words=1 tile=64x64 a=4096 b=4096 outer=0 "), tp.last_plan()
    got = out.cpu().numpy()
    assert np.array_equal(got[8:].view(np.float64).reshape(n, n), a_h.T) and not got[:8].any()
    few = 64 * n * 8   # the first 64 columns through the oracle as well
    expect = np.zeros(few, np.uint8)
    cc.pack(a_h.reshape(-1).view(np.uint8), 0, 1, hvector(64, 1, 8, vector(n, 1, n, DOUBLE)), expect, 0)
    assert np.array_equal(got[8:8 + few], expect)
    say("full-size transpose: unpack")
    back = torch.full((n * n * 8,), 0xA5, dtype=torch.uint8, device=dev)
    assert tp.unpack(out, size + 8, 8, back, 1, h) == size + 8
    assert torch.equal(back, a)


def test_sixteen_dimensions(dev):
    # 15 nested two-element levels and two objects: 16 row dimensions, the most a launch carries
    say("sixteen dimensions")
    t = contiguous(3, BYTE)
    stride = 4
    for _ in range(15):
        t = hvector(2, 1, stride, t)
        stride = 2 * stride + 1
    roundtrip(t, 2, dev, typed_shift=1, seed=16)
    assert "nrd=16" in tp.last_plan()


def test_word_widths_forced(dev):
    t = vector(300, 64, 96, BYTE)
    try:
        for w in (1, 2, 4, 8, 16):
            say("forced word", w)
            tp.set_override("word", w)
            plans = roundtrip(t, 2, dev, seed=w)
            assert f"W={w} " in plans["pack"] and f"W={min(w, 8)} ux=1 ur=1 nt=7 " in plans["unpack"]
            # rows of whole 64-byte segments: the unpack may use the wide words too
            plans = roundtrip(vector(300, 192, 256, BYTE), 2, dev, seed=w)
            assert f"W={w} " in plans["pack"] and f"W={w} " in plans["unpack"]
    finally:
        tp.set_override("word", 0)


def test_launch_splitting_on_gpu(dev):
    t = hvector(7, 1, 4096, hvector(5, 1, 512, vector(9, 16, 32, BYTE)))
    try:
        tp.set_override("max_rows_per_launch", 11)
        tp.set_override("max_words_per_run", 3)
        say("split launches")
        roundtrip(t, 3, dev, seed=5)
        assert tp.last_plan().count("\n") > 10
    finally:
        tp.set_override("max_rows_per_launch", 1 << 30)
        tp.set_override("max_words_per_run", 1 << 30)


def test_empty_and_degenerate(dev):
    say("empty / degenerate")
    buf = torch.zeros(64, dtype=torch.uint8, device=dev)
    out = torch.full((64,), 7, dtype=torch.uint8, device=dev)
    empty = tp.type_from_recipe(vector(0, 2, 4, BYTE))
    assert tp.pack(buf, 5, empty, out, 64, 9) == 9
    one = tp.type_from_recipe(contiguous(1, BYTE))
    assert tp.pack(buf, 0, one, out, 64, 9) == 9
    assert tp.pack(buf, 1, one, out, 10, 9) == 10           # exactly fits
    with pytest.raises(tp.TpError) as e:
        tp.pack(buf, 2, one, out, 10, 9)
    assert e.value.code == tp.TP_ERR_TRUNCATE
    assert (out.cpu().numpy()[10:] == 7).all()
    roundtrip(BYTE, 1, dev)
    roundtrip(DOUBLE, 7, dev, typed_shift=8)
    roundtrip(contiguous(1 << 20, BYTE), 1, dev, typed_shift=1, packed_shift=3)   # unaligned plain copy
    # the origin handed to pack may lie outside the allocation as long as the selected bytes do not
    say("origin before the allocation")
    sub = tp.type_from_recipe(subarray((8, 512), (2, 16), (4, 0), "C", BYTE))   # first byte at +2048
    data_h = W.random_bytes(8, 1024)
    data = to_dev(data_h, dev)
    out2 = torch.zeros(32, dtype=torch.uint8, device=dev)
    assert tp.pack(data.data_ptr() - 2048, 1, sub, out2, 32, 0) == 32
    assert np.array_equal(out2.cpu().numpy(), np.concatenate([data_h[0:16], data_h[512:528]]))


def test_pageable_host_memory_is_rejected(dev):
    host = np.zeros(64, dtype=np.uint8)
    out = torch.zeros(64, dtype=torch.uint8, device=dev)
    t = tp.type_from_recipe(vector(3, 2, 4, BYTE))
    with pytest.raises(tp.TpError) as e:
        tp.pack(host.ctypes.data, 1, t, out, 64, 0)
    assert e.value.code == tp.TP_ERR_BUFFER
    pinned = torch.zeros(64, dtype=torch.uint8).pin_memory()
    with pytest.raises(tp.TpError) as e:   # the typed side must be device memory
        tp.pack(pinned, 1, t, out, 64, 0)
    assert e.value.code == tp.TP_ERR_BUFFER
    # the library still works afterwards
    roundtrip(vector(3, 2, 4, BYTE), 1, dev)


# ------------------------------------------------------------------ the five workloads
def test_cfg1_both_constructions(dev):
    c = W.configs.cfg1()
    src_h = W.random_bytes(c["seed"], c["buffer_bytes"])
    src = to_dev(src_h, dev)
    outs = []
    for name, r in c["recipes"].items():
        say("cfg1", name)
        h = tp.type_from_recipe(r)
        assert tp.type_get_strided_block(h) == (0, [8, 64], [1, 512])
        out = torch.zeros(512, dtype=torch.uint8, device=dev)
        assert tp.pack(src, 1, h, out, 512, 0) == 512
        expect = np.zeros(512, np.uint8)
        cc.pack(src_h, 0, 1, r, expect, 0)
        assert np.array_equal(out.cpu().numpy(), expect)
        assert np.array_equal(expect, src_h[:64 * 512].reshape(64, 512)[:, :8].reshape(-1))
        back = torch.full((c["buffer_bytes"],), 0xA5, dtype=torch.uint8, device=dev)
        assert tp.unpack(out, 512, 0, back, 1, h) == 512
        want = np.full(c["buffer_bytes"], 0xA5, np.uint8)
        cc.unpack(expect, 0, want, 0, 1, r)
        assert np.array_equal(back.cpu().numpy(), want)
        outs.append(expect)
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("a0", W.configs.A0_SWEEP)
def test_cfg2_1mib_full(dev, a0):
    p = W.configs.cfg2_point(a0, 1 << 20)
    say("cfg2 1MiB a0", a0, p["a"], "alloc", p["alloc_bytes"] >> 20, "MiB")
    src = W.fills.counter_bytes_torch(p["seed"], p["alloc_bytes"], dev)
    src_h = src.cpu().numpy()
    h = tp.type_from_recipe(p["recipe"])
    out = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    assert tp.pack(src, 1, h, out, 1 << 20, 0) == 1 << 20
    expect = np.zeros(1 << 20, np.uint8)
    cc.pack(src_h, 0, 1, p["recipe"], expect, 0, nthreads=8)
    assert np.array_equal(out.cpu().numpy(), expect), tp.last_plan()
    a0_, a1, a2 = p["a"]
    assert np.array_equal(expect, src_h.reshape(-1, 512, 512)[:a2, :a1, :a0].reshape(-1))
    back = torch.full((p["alloc_bytes"],), 0xA5, dtype=torch.uint8, device=dev)
    assert tp.unpack(out, 1 << 20, 0, back, 1, h) == 1 << 20
    want = np.full(p["alloc_bytes"], 0xA5, np.uint8)
    cc.unpack(expect, 0, want, 0, 1, p["recipe"], nthreads=8)
    assert torch.equal(back.cpu(), torch.from_numpy(want)), tp.last_plan()


@pytest.mark.parametrize("a0", W.configs.A0_SWEEP)
def test_cfg2_64mib_full(dev, a0):
    # The benchmark's own size and launch configuration, every byte compared.  The typed allocation
    # reaches 32 GiB and never exists on the host: the fill is a counter-based stream, so the byte
    # that the oracle's type map names for packed position k is computed on the host for every k.
    p = W.configs.cfg2_point(a0, 1 << 26)
    say("cfg2 64MiB a0", a0, p["a"], "alloc", p["alloc_bytes"] >> 20, "MiB")
    src = W.fills.counter_bytes_torch(p["seed"], p["alloc_bytes"], dev)
    h = tp.type_from_recipe(p["recipe"])
    n = 1 << 26
    out = torch.zeros(n, dtype=torch.uint8, device=dev)
    assert tp.pack(src, 1, h, out, n, 0) == n
    plan = tp.last_plan()
    got = out.cpu().numpy()
    del src
    say("  oracle type map")
    d, ln = cc.blocks(p["recipe"])            # the C oracle's own (displacement, length) blocks, in packed order
    assert int(ln.sum()) == n
    ends = np.cumsum(ln)
    step = 1 << 22
    for lo in range(0, d.size, step):
        dd, ll = d[lo:lo + step], ln[lo:lo + step]
        first = int(ends[lo] - ln[lo])
        total = int(ll.sum())
        # displacement of every byte of these blocks: block start + offset within the block
        disp = dd if total == dd.size else np.repeat(dd, ll) + (np.arange(total) - np.repeat(np.cumsum(ll) - ll, ll))
        assert np.array_equal(got[first:first + total], W.fills.counter_byte_at(p["seed"], disp)), (lo, plan)
    del d, ln, ends
    # Unpack into a poisoned allocation and compare all of it on the device against an expectation that
    # owes nothing to the library or the oracle: the allocation seen as an e2 x 512 x 512 array, the
    # selected box [0:a2, 0:a1, 0:a0] of it must be the packed stream reshaped, and outside the box
    # nothing may differ from the poison (as many bytes differ from it in the whole allocation as in
    # the packed stream itself).
    say("  unpack")
    a0_, a1, a2 = p["a"]
    e2 = p["e"][2]
    back = torch.full((p["alloc_bytes"],), 0xA5, dtype=torch.uint8, device=dev)
    assert tp.unpack(out, n, 0, back, 1, h) == n
    plan = tp.last_plan()
    vol = back.view(e2, 512, 512)
    box = out.view(a2, a1, a0_)
    planes = 4096                                  # 1 GiB of the allocation at a time
    differ = 0
    for z0 in range(0, e2, planes):
        z1 = min(e2, z0 + planes)
        differ += int((vol[z0:z1] != 0xA5).sum().item())
        if z0 < a2:
            zb = min(a2, z1)
            assert torch.equal(vol[z0:zb, :a1, :a0_], box[z0:zb]), (z0, plan)
    assert differ == int((out != 0xA5).sum().item()), plan


def test_cfg3_halo_full(dev):
    c = W.configs.cfg3()
    say("cfg3 generating grid")
    grid_h = W.random_grid_f64(c["seed"], c["grid_shape"])
    raw_h = grid_h.reshape(-1).view(np.uint8)
    grid = to_dev(raw_h, dev)
    send = [tp.type_from_recipe(r) for r in c["send"]]
    ghost = [tp.type_from_recipe(r) for r in c["ghost_for_send"]]
    total = sum(tp.type_size(h) for h in send)
    assert total == 37308096
    packed = torch.zeros(total, dtype=torch.uint8, device=dev)
    pos = 0
    expect = np.zeros(total, np.uint8)
    epos = 0
    for i, (h, r) in enumerate(zip(send, c["send"])):
        say("cfg3 pack", i, c["directions"][i])
        pos = tp.pack(grid, 1, h, packed, total, pos)
        epos = cc.pack(raw_h, 0, 1, r, expect, epos)
        assert pos == epos
    assert pos == total
    assert np.array_equal(packed.cpu().numpy(), expect)
    # numpy slices as a third opinion on the first and last regions
    for i in (0, 12, 25):
        reg = c["send_region"][i]
        sel = np.ascontiguousarray(grid_h[tuple(slice(a, b) for a, b in reg)]).reshape(-1).view(np.uint8)
        off = sum(tp.type_size(h) for h in send[:i])
        assert np.array_equal(expect[off:off + sel.size], sel)
    # unpack every message into the ghost zone of the opposite direction
    pos = 0
    epos = 0
    want = raw_h.copy()
    for i, (h, r) in enumerate(zip(ghost, c["ghost_for_send"])):
        say("cfg3 unpack", i)
        pos = tp.unpack(packed, total, pos, grid, 1, h)
        epos = cc.unpack(expect, epos, want, 0, 1, r)
    assert pos == epos == total
    got = grid.cpu().numpy()
    assert np.array_equal(got, want)
    g = got.view(np.float64).reshape(c["grid_shape"])
    for i in (0, 13, 25):   # periodic self-exchange: ghost(-d) now equals the interior send(d)
        s_reg, g_reg = c["send_region"][i], c["ghost_region_for_send"][i]
        assert np.array_equal(g[tuple(slice(a, b) for a, b in g_reg)], grid_h[tuple(slice(a, b) for a, b in s_reg)])


@pytest.mark.parametrize("bl", W.configs.CFG4_BLOCKLENGTHS)
def test_cfg4_tiny_runs_full(dev, bl):
    p = W.configs.cfg4_point(bl)
    src = W.fills.counter_bytes_torch(p["seed"], p["source_bytes"], dev)
    src_h = src.cpu().numpy()
    n = p["packed_bytes"]
    h = tp.type_from_recipe(p["recipe"])
    for k in W.configs.CFG4_OFFSETS:
        for position in ((0, 1) if k in (0, 5) else (0,)):
            say("cfg4 bl", bl, "offset", k, "position", position)
            out = torch.zeros(n + position, dtype=torch.uint8, device=dev)
            assert tp.pack(src.data_ptr() + k, 1, h, out, n + position, position) == n + position
            expect = np.ascontiguousarray(src_h[k:k + (1 << 24) * 64].reshape(-1, 64)[:, :bl]).reshape(-1)
            got = out.cpu().numpy()
            assert np.array_equal(got[position:], expect), tp.last_plan()
            if k in (0, 3):
                ref = np.zeros(n, np.uint8)
                cc.pack(src_h, k, 1, p["recipe"], ref, 0, nthreads=8)
                assert np.array_equal(ref, expect)
            if k in (0, 5):
                back = torch.full((p["source_bytes"],), 0xA5, dtype=torch.uint8, device=dev)
                assert tp.unpack(out, n + position, position, back.data_ptr() + k, 1, h) == n + position
                b = back.cpu().numpy()
                rows = b[k:k + (1 << 24) * 64].reshape(-1, 64)
                assert np.array_equal(rows[:, :bl].reshape(-1), expect)
                assert (rows[:, bl:] == 0xA5).all() and (b[:k] == 0xA5).all() and (b[k + (1 << 30):] == 0xA5).all()
    # the same layout with the offset inside the type (subarray start)
    hs = tp.type_from_recipe(p["recipe_subarray"](5))
    out = torch.zeros(n, dtype=torch.uint8, device=dev)
    tp.pack(src, 1, hs, out, n, 0)
    assert np.array_equal(out.cpu().numpy(), np.ascontiguousarray(src_h[5:5 + (1 << 30)].reshape(-1, 64)[:, :bl]).reshape(-1))


def test_cfg5_nested_batch(dev):
    c = W.configs.cfg5()
    r = c["recipe"]
    h = tp.type_from_recipe(r)
    ex = tp.type_get_extent(h)[1]
    size = tp.type_size(h)
    nobj = c["objects"]
    say("cfg5 generating", nobj * ex >> 20, "MiB")
    src = W.fills.counter_bytes_torch(c["seed"], nobj * ex, dev)
    out = torch.zeros(nobj * size, dtype=torch.uint8, device=dev)
    say("cfg5 one call, incount", nobj)
    assert tp.pack(src, nobj, h, out, nobj * size, 0) == nobj * size
    src_h = src.cpu().numpy()
    expect = np.zeros(nobj * size, np.uint8)
    say("cfg5 oracle")
    cc.pack(src_h, 0, nobj, r, expect, 0, nthreads=16)
    assert np.array_equal(out.cpu().numpy(), expect), tp.last_plan()
    # 1000 enqueue-only calls and one synchronize
    say("cfg5 async calls")
    out.zero_()
    pos = 0
    for i in range(nobj):
        pos = tp.pack_async(src.data_ptr() + i * ex, 1, h, out, nobj * size, pos)
    torch.cuda.synchronize()
    assert pos == nobj * size
    assert np.array_equal(out.cpu().numpy(), expect)
    # zero-copy: the packed stream written straight into pinned host memory
    say("cfg5 pinned host")
    few = 64
    pinned = torch.zeros(few * size, dtype=torch.uint8).pin_memory()
    assert tp.pack(src, few, h, pinned, few * size, 0) == few * size
    assert np.array_equal(pinned.numpy(), expect[:few * size])


def test_pinned_host_packed_side(dev):
    say("pinned packed side, small types")
    roundtrip(vector(1031, 24, 40, BYTE), 2, dev, pinned_packed=True, seed=3)
    roundtrip(hvector(37, 1, 20480, contiguous(4100, BYTE)), 1, dev, pinned_packed=True, packed_shift=4, seed=4)
    # unaligned 16-byte accesses to mapped host memory: odd address, odd run length
    roundtrip(hvector(37, 1, 20480, contiguous(4099, BYTE)), 2, dev, pinned_packed=True, packed_shift=3, typed_shift=1,
              position=5, seed=5)
    roundtrip(vector(1031, 21, 40, BYTE), 2, dev, pinned_packed=True, packed_shift=1, seed=6)
    # unpack from pinned host memory as well
    t = vector(513, 16, 48, BYTE)
    h = tp.type_from_recipe(t)
    size = tp.type_size(h)
    ex = tp.type_get_extent(h)[1]
    packed_h = W.random_bytes(9, size)
    pinned = torch.from_numpy(packed_h).pin_memory()
    dst = torch.full((ex,), 0xA5, dtype=torch.uint8, device=dev)
    assert tp.unpack(pinned, size, 0, dst, 1, h) == size
    want = np.full(ex, 0xA5, np.uint8)
    cc.unpack(packed_h, 0, want, 0, 1, t)
    assert np.array_equal(dst.cpu().numpy(), want)
    # ... from an odd address in it, rows of odd length into an odd typed address
    t = hvector(29, 1, 9001, contiguous(4099, BYTE))
    h = tp.type_from_recipe(t)
    size, ex = tp.type_size(h), tp.type_get_extent(h)[1]
    packed_h = W.random_bytes(10, size + 7)
    pinned = torch.from_numpy(packed_h).pin_memory()
    dst = torch.full((ex + 3,), 0xA5, dtype=torch.uint8, device=dev)
    assert tp.unpack(pinned.data_ptr() + 3, size + 4, 4, dst.data_ptr() + 3, 1, h) == size + 4
    want = np.full(ex + 3, 0xA5, np.uint8)
    cc.unpack(packed_h[3:], 4, want, 3, 1, t)
    assert np.array_equal(dst.cpu().numpy(), want)


def test_counter_fill_matches_on_device(dev):
    a = W.fills.counter_bytes_torch(77, 100003, dev, chunk_words=4099).cpu().numpy()
    assert np.array_equal(a, W.fills.counter_bytes_numpy(77, 0, 100003))


# ------------------------------------------------------------------ batched calls
def test_batch_halo_equals_separate_calls(dev):
    # all 26 regions in one tp_pack_batch / tp_unpack_batch, against the oracle and the per-call path
    c = W.configs.cfg3()
    grid_h = W.random_grid_f64(c["seed"] + 100, c["grid_shape"])
    raw_h = grid_h.reshape(-1).view(np.uint8)
    grid = to_dev(raw_h, dev)
    send = [tp.type_from_recipe(r) for r in c["send"]]
    ghost = [tp.type_from_recipe(r) for r in c["ghost_for_send"]]
    total = sum(tp.type_size(h) for h in send)
    packed = torch.zeros(total + 8, dtype=torch.uint8, device=dev)
    say("batch halo pack")
    b = tp.Batch([grid] * 26, [1] * 26, send)
    assert tp.pack_batch(b, packed, total + 8, 8) == total + 8
    plan = tp.last_plan()
    assert plan.count("batch") == 1 and "tile" not in plan, plan
    expect = np.zeros(total + 8, np.uint8)
    pos = 8
    for r in c["send"]:
        pos = cc.pack(raw_h, 0, 1, r, expect, pos)
    assert np.array_equal(packed.cpu().numpy(), expect)
    say("batch halo unpack")
    g = tp.Batch([grid] * 26, [1] * 26, ghost)
    assert tp.unpack_batch(packed, total + 8, 8, g) == total + 8
    want = raw_h.copy()
    pos = 8
    for r in c["ghost_for_send"]:
        pos = cc.unpack(expect, pos, want, 0, 1, r)
    assert np.array_equal(grid.cpu().numpy(), want)


def test_batch_mixed_types_and_fallback(dev):
    # 70 random types (some with too many dimensions for a batch descriptor) in one call
    rng = random.Random(501)
    reqs = []
    typed_len = 0
    while len(reqs) < 70:
        t = W.random_recipe(rng, rng.randint(1, 4))
        if py.size(t) > 4096:
            continue
        count = rng.randint(1, 3)
        if py.has_overlap(t, count):
            continue
        d, n = cc.blocks(t, count)
        origin = typed_len + rng.choice((0, 1, 2, 4, 8, 16))
        typed_len = origin + int((d + n).max()) + 16
        reqs.append((t, count, origin))
    deep = hvector(2, 1, 100000, hvector(3, 1, 30000, hvector(2, 1, 14000, vector(3, 2, 100, hvector(2, 1, 40, named("INT16"))))))
    assert not py.has_overlap(deep, 2)
    reqs.insert(30, (deep, 2, typed_len))
    typed_len += 2 * cc.extent(deep) + 16
    # and a matrix walked by columns, which the transposing kernel takes (never part of a batch)
    walked = hvector(70, 1, 8, vector(45, 1, 70, DOUBLE))
    reqs.insert(50, (walked, 2, typed_len + 3))
    typed_len += 3 + 2 * cc.extent(walked) + 16
    typed_h = W.random_bytes(6, typed_len)
    typed = to_dev(typed_h, dev)
    handles = [tp.type_from_recipe(t) for t, _, _ in reqs]
    total = sum(tp.type_size(h) * c for h, (_, c, _) in zip(handles, reqs))
    packed = torch.full((total + 5,), 0xEE, dtype=torch.uint8, device=dev)
    say("batch mixed pack")
    b = tp.Batch([typed.data_ptr() + o for _, _, o in reqs], [c for _, c, _ in reqs], handles)
    assert tp.pack_batch(b, packed, total + 5, 5) == total + 5
    plan = tp.last_plan()
    assert plan.count("batch") == 2 and plan.count("tile") >= 1 and plan.count("xpose") == 1, plan
    expect = np.full(total + 5, 0xEE, np.uint8)
    pos = 5
    for t, c, o in reqs:
        pos = cc.pack(typed_h, o, c, t, expect, pos)
    assert np.array_equal(packed.cpu().numpy(), expect)
    say("batch mixed unpack")
    back = torch.full((typed_len,), 0xA5, dtype=torch.uint8, device=dev)
    bb = tp.Batch([back.data_ptr() + o for _, _, o in reqs], [c for _, c, _ in reqs], handles)
    assert tp.unpack_batch(packed, total + 5, 5, bb) == total + 5
    want = np.full(typed_len, 0xA5, np.uint8)
    pos = 5
    for t, c, o in reqs:
        pos = cc.unpack(expect, pos, want, o, c, t)
    assert np.array_equal(back.cpu().numpy(), want)
    # an invalid request anywhere: nothing is written, the position does not move
    packed.fill_(0x11)
    bad = tp.Batch([typed.data_ptr()] * 3, [1, 1, 1], [handles[0], 999999, handles[1]])
    with pytest.raises(tp.TpError) as e:
        tp.pack_batch(bad, packed, total + 5, 0)
    assert e.value.code == tp.TP_ERR_TYPE
    assert (packed.cpu().numpy() == 0x11).all()


def test_batch_unpack_large_requests_take_their_own_launch(dev):
    # small requests ride in the batched launch; requests of 2^20 rows or 8 MiB that write through get
    # a launch of their own (one row per thread, sc1 nt stores); the bytes are the oracle's either way
    reqs, typed_len = [], 0
    for t in (vector(300, 24, 64, BYTE), vector((1 << 20) + 5, 3, 16, BYTE), vector(100, 200, 512, BYTE),
              vector(45000, 200, 512, BYTE), hvector(7, 1, 5000, vector(40, 10, 100, BYTE)),
              vector((1 << 20) + 9, 4, 512, BYTE)):
        d, n = cc.blocks(t, 1)
        origin = typed_len + 1
        typed_len = origin + int((d + n).max()) + 16
        reqs.append((t, 1, origin))
    handles = [tp.type_from_recipe(t) for t, _, _ in reqs]
    total = sum(tp.type_size(h) for h in handles)
    packed_h = W.random_bytes(11, total + 3)
    packed = to_dev(packed_h, dev)
    back = torch.full((typed_len,), 0xA5, dtype=torch.uint8, device=dev)
    say("batch unpack, small and large requests", total, "bytes")
    bb = tp.Batch([back.data_ptr() + o for _, _, o in reqs], [1] * len(reqs), handles)
    assert tp.unpack_batch(packed, total + 3, 3, bb) == total + 3
    plan = tp.last_plan()
    assert plan.count("batch") == 1 and plan.count("ur=1 nt=7") == 2 and "rows=1048581" in plan and "rows=45000" in plan, plan
    assert plan.count("prefetch") == 1 and "tile W=4 ux=1 ur=1 nt=6 bx=1 n0=1 back=0 rows=1048585 " in plan, plan   # and staged
    want = np.full(typed_len, 0xA5, np.uint8)
    pos = 3
    for t, c, o in reqs:
        pos = cc.unpack(packed_h, pos, want, o, c, t)
    assert np.array_equal(back.cpu().numpy(), want)


def test_batch_many_objects_of_one_type(dev):
    # 300 separately addressed objects of the nested 4-level type: 8 batched launches instead of 300
    c = W.configs.cfg5()
    r = c["recipe"]
    h = tp.type_from_recipe(r)
    ex, size, nobj = tp.type_get_extent(h)[1], tp.type_size(h), 300
    src = W.fills.counter_bytes_torch(c["seed"] + 7, nobj * ex, dev)
    src_h = src.cpu().numpy()
    out = torch.zeros(nobj * size, dtype=torch.uint8, device=dev)
    order = list(range(nobj))
    random.Random(3).shuffle(order)
    say("batch 300 objects")
    b = tp.Batch([src.data_ptr() + i * ex for i in order], [1] * nobj, [h] * nobj)
    assert tp.pack_batch_async(b, out, nobj * size, 0) == nobj * size
    torch.cuda.synchronize()
    assert tp.last_plan().count("batch") == 8
    expect = np.zeros(nobj * size, np.uint8)
    pos = 0
    for i in order:
        pos = cc.pack(src_h, i * ex, 1, r, expect, pos)
    assert np.array_equal(out.cpu().numpy(), expect)


def test_async_calls_replay_from_a_hip_graph(dev):
    # the enqueue-only entry points allocate nothing and record no memset, so a stream capture of
    # them replays correctly: capture the 26 halo packs once, replay after changing the grid
    c = W.configs.cfg3(32, 3)
    n = 32
    send = [tp.type_from_recipe(r) for r in c["send"]]
    total = sum(tp.type_size(h) for h in send)
    grid = torch.zeros(n * n * n * 8, dtype=torch.uint8, device=dev)
    packed = torch.zeros(total, dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    say("capture 26 pack_async calls")
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        pos = 0
        for h in send:
            pos = tp.pack_async(grid, 1, h, packed, total, pos, torch.cuda.current_stream())
    assert pos == total
    for rep in range(4):
        say("replay", rep)
        grid_h = W.random_grid_f64(700 + rep, (n, n, n)).reshape(-1).view(np.uint8)
        grid.copy_(torch.from_numpy(grid_h))       # eager work between replays
        packed.fill_(0x5A)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        expect = np.zeros(total, np.uint8)
        p = 0
        for r in c["send"]:
            p = cc.pack(grid_h, 0, 1, r, expect, p)
        assert np.array_equal(packed.cpu().numpy(), expect)


def test_staged_unpack_replays_from_a_hip_graph(dev):
    # a staged unpack is several launches (read-only passes and store passes): captured once, it replays
    # with new packed bytes each time
    rows, run, pitch = (1 << 20) + 700, 4, 256
    t = vector(rows, run, pitch, BYTE)
    h = tp.type_from_recipe(t)
    size = rows * run
    packed = torch.zeros(size, dtype=torch.uint8, device=dev)
    typed = torch.full((rows * pitch + 64,), 0xA5, dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    say("capture a staged unpack")
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        assert tp.unpack_async(packed, size, 0, typed.data_ptr() + 8, 1, h, torch.cuda.current_stream()) == size
    assert tp.last_plan().count("prefetch") == 1 and tp.last_plan().count("tile W=4 ux=1 ur=1 nt=6") == 2, tp.last_plan()
    for rep in range(3):
        say("replay", rep)
        packed_h = W.random_bytes(900 + rep, size)
        packed.copy_(torch.from_numpy(packed_h))     # eager work between replays
        typed.fill_(0xA5)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want = np.full(rows * pitch + 64, 0xA5, np.uint8)
        cc.unpack(packed_h, 0, want, 8, 1, t)
        assert np.array_equal(typed.cpu().numpy(), want)


# ------------------------------------------------------------------ model and host delivery
def test_model_measure_and_host_delivery(dev, tmp_path):
    from oracle import model as om
    say("tp_model_measure")
    tp.model_measure()
    path = tmp_path / "model.txt"
    tp.model_save(str(path))
    table = om.parse(path.read_text())
    for name in om.PRIMITIVES:
        assert (table[name] > 0).all() and (table[name] < 1.0).all(), name
    # the largest objects cost more than the smallest, and every call has a latency floor above 1 us
    assert (table["gpu_pack"][-1] > table["gpu_pack"][0]).all() and table["gpu_pack"].min() > 1e-6
    assert table["d2h"][-1] > table["d2h"][0]
    # the library's interpolation of its own measured table equals the oracle's
    t = vector(5000, 24, 512, BYTE)
    h = tp.type_from_recipe(t)
    size = tp.type_size(h)
    want = om.query(table, size * 3, 24)
    got = tp.model_query(h, 3)
    assert all(abs(got[k] - want[k]) <= 1e-12 * want[k] for k in want)
    m, totals = tp.model_select(h, 3)
    assert (m, totals) == (om.select(want)[0], pytest.approx(om.select(want)[1], rel=1e-12))

    ex = tp.type_get_extent(h)[1]
    src_h = W.random_bytes(21, ex * 3)
    src = to_dev(src_h, dev)
    expect = np.full(size * 3 + 4, 0xEE, np.uint8)
    cc.pack(src_h, 0, 3, t, expect, 4)
    staging = torch.zeros(size * 3, dtype=torch.uint8, device=dev)
    for method in (tp.TP_METHOD_ONESHOT, tp.TP_METHOD_STAGED, tp.TP_METHOD_AUTO):
        say("pack_host method", method)
        host = torch.full((size * 3 + 4,), 0xEE, dtype=torch.uint8).pin_memory()
        pos, used = tp.pack_host(src, 3, h, host, size * 3 + 4, 4, staging, size * 3, method)
        assert pos == size * 3 + 4 and used in (tp.TP_METHOD_ONESHOT, tp.TP_METHOD_STAGED)
        if method != tp.TP_METHOD_AUTO:
            assert used == method
        else:
            assert used == (tp.TP_METHOD_STAGED if want["gpu_pack"] + want["d2h"] < want["host_pack"]
                            else tp.TP_METHOD_ONESHOT)
        assert np.array_equal(host.numpy(), expect)
        back = torch.full((ex * 3,), 0xA5, dtype=torch.uint8, device=dev)
        pos, used = tp.unpack_host(host, size * 3 + 4, 4, back, 3, h, staging, size * 3, method)
        assert pos == size * 3 + 4
        wantb = np.full(ex * 3, 0xA5, np.uint8)
        cc.unpack(expect, 4, wantb, 0, 3, t)
        assert np.array_equal(back.cpu().numpy(), wantb)
    # staged without a large enough staging buffer is an argument error; auto falls back to one-shot
    host = torch.zeros(size * 3, dtype=torch.uint8).pin_memory()
    with pytest.raises(tp.TpError) as e:
        tp.pack_host(src, 3, h, host, size * 3, 0, staging, 10, tp.TP_METHOD_STAGED)
    assert e.value.code == tp.TP_ERR_ARG
    assert tp.pack_host(src, 3, h, host, size * 3, 0, None, 0, tp.TP_METHOD_AUTO) == (size * 3, tp.TP_METHOD_ONESHOT)
    assert np.array_equal(host.numpy(), expect[4:])


def test_datatype_running_past_its_buffer_is_refused(dev):
    # the lowest and highest byte of a request must be memory the GPU can address; a type that
    # leaves its buffer is an error on the host, not a fault on the device
    far = 1 << 44  # 16 TiB: no allocation of this process reaches that far
    buf = torch.zeros(4096, dtype=torch.uint8, device=dev)
    out = torch.full((4096,), 0xEE, dtype=torch.uint8, device=dev)
    for name, recipe in (("above", hvector(2, 1, far, BYTE)), ("below", hvector(2, 1, -far, BYTE)),
                         ("objects", subarray([1 << 30, 1 << 14], [1, 1], [0, 0], "C", BYTE))):
        h = tp.type_from_recipe(recipe)
        count = 1 if name != "objects" else 2  # one byte per object, the second object 2^44 bytes on
        say("span check:", name)
        for fn, args in ((tp.pack, (buf, count, h, out, 1 << 62, 0)), (tp.unpack, (out, 1 << 62, 0, buf, count, h))):
            with pytest.raises(tp.TpError) as e:
                fn(*args)
            assert e.value.code == tp.TP_ERR_BUFFER
    # the contiguous side: a position far beyond the buffer
    h = tp.type_from_recipe(contiguous(2, BYTE))
    for fn, args in ((tp.pack, (buf, 1, h, out, far + 2, far)), (tp.unpack, (out, far + 2, far, buf, 1, h))):
        with pytest.raises(tp.TpError) as e:
            fn(*args)
        assert e.value.code == tp.TP_ERR_BUFFER
    torch.cuda.synchronize()
    assert bool((out == 0xEE).all()) and bool((buf == 0).all())


# ------------------------------------------------------------------ resource cache
class _DeviceView:
    """Zero-copy torch view of `n` bytes of device memory at `address` (owned elsewhere)."""

    def __init__(self, address, n):
        self.__cuda_array_interface__ = {"shape": (n,), "typestr": "|u1", "data": (address, False), "version": 2}


def _host_view(address, n):
    import ctypes
    return np.ctypeslib.as_array((ctypes.c_uint8 * n).from_address(address))


def test_resource_cache_buffers_serve_pack_and_unpack(dev):
    t = hvector(40, 1, 5000, vector(19, 3, 7, named("INT16")))
    h = tp.type_from_recipe(t)
    size, ex = tp.type_size(h), tp.type_get_extent(h)[1]
    src_h = W.random_bytes(501, ex)
    src = to_dev(src_h, dev)
    expect = np.zeros(size, np.uint8)
    cc.pack(src_h, 0, 1, t, expect, 0)
    before = {k: tp.resource_stats(k) for k in range(4)}

    say("resource cache: device buffer as the packed side")
    d = tp.resource_acquire(tp.TP_RES_DEVICE, size)
    assert d % 256 == 0
    assert tp.pack(src, 1, h, d + 2, size, 0) == size  # an odd offset inside the lease
    got = torch.as_tensor(_DeviceView(d, size + 2), device=dev).cpu().numpy()
    assert np.array_equal(got[2:], expect)

    say("resource cache: pinned buffer as the packed side, both directions")
    p = tp.resource_acquire(tp.TP_RES_PINNED, size)
    host = _host_view(p, size)
    host[:] = 0
    assert tp.pack(src, 1, h, p, size, 0) == size
    assert np.array_equal(host, expect)
    back = torch.full((ex,), 0xA5, dtype=torch.uint8, device=dev)
    assert tp.unpack(p, size, 0, back, 1, h) == size
    want = np.full(ex, 0xA5, np.uint8)
    cc.unpack(expect, 0, want, 0, 1, t)
    assert np.array_equal(back.cpu().numpy(), want)
    # a leased pinned buffer is still host memory: not acceptable as the typed side
    with pytest.raises(tp.TpError) as e:
        tp.pack(p, 1, tp.type_from_recipe(contiguous(16, BYTE)), d, size, 0)
    assert e.value.code == tp.TP_ERR_BUFFER

    say("resource cache: stream and event from the cache")
    s = tp.resource_acquire(tp.TP_RES_STREAM)
    ev = tp.resource_acquire(tp.TP_RES_EVENT)
    out = torch.zeros(size, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    assert tp.pack(src, 1, h, out, size, 0, s) == size  # synchronizes on s
    assert np.array_equal(out.cpu().numpy(), expect)

    say("resource cache: release, reuse, trim")
    for kind, handle in ((tp.TP_RES_DEVICE, d), (tp.TP_RES_PINNED, p), (tp.TP_RES_STREAM, s), (tp.TP_RES_EVENT, ev)):
        tp.resource_release(kind, handle)
        with pytest.raises(tp.TpError) as e:
            tp.resource_release(kind, handle)
        assert e.value.code == tp.TP_ERR_ARG
        again = tp.resource_acquire(kind, size)
        assert again == handle
        tp.resource_release(kind, again)
        now = tp.resource_stats(kind)
        assert now["misses"] - before[kind]["misses"] == 1 and now["hits"] - before[kind]["hits"] == 1
        assert now["leased"] == before[kind]["leased"] and now["idle"] == before[kind]["idle"] + 1
    idle = tp.resource_stats(tp.TP_RES_DEVICE)["idle_bytes"] + tp.resource_stats(tp.TP_RES_PINNED)["idle_bytes"]
    assert tp.resource_trim() == idle and tp.resource_trim() == 0
    assert all(tp.resource_stats(k)["idle"] == 0 for k in range(4))


def test_staged_host_delivery_with_cached_staging(dev):
    t = vector(3000, 40, 96, BYTE)
    h = tp.type_from_recipe(t)
    size, ex = tp.type_size(h), tp.type_get_extent(h)[1]
    src_h = W.random_bytes(502, ex * 2)
    src = to_dev(src_h, dev)
    expect = np.full(size * 2 + 8, 0xEE, np.uint8)
    cc.pack(src_h, 0, 2, t, expect, 8)
    tp.resource_trim()
    start = tp.resource_stats(tp.TP_RES_DEVICE)
    for i in range(3):
        say("staged delivery without a staging buffer, call", i)
        host = torch.full((size * 2 + 8,), 0xEE, dtype=torch.uint8).pin_memory()
        assert tp.pack_host(src, 2, h, host, size * 2 + 8, 8, None, 0, tp.TP_METHOD_STAGED) == \
            (size * 2 + 8, tp.TP_METHOD_STAGED)
        assert np.array_equal(host.numpy(), expect)
        back = torch.full((ex * 2,), 0xA5, dtype=torch.uint8, device=dev)
        assert tp.unpack_host(host, size * 2 + 8, 8, back, 2, h, None, 0, tp.TP_METHOD_STAGED) == \
            (size * 2 + 8, tp.TP_METHOD_STAGED)
        want = np.full(ex * 2, 0xA5, np.uint8)
        cc.unpack(expect, 8, want, 0, 2, t)
        assert np.array_equal(back.cpu().numpy(), want)
    end = tp.resource_stats(tp.TP_RES_DEVICE)
    # six staged transfers: one allocation, five served from the cache, nothing left leased
    assert end["misses"] - start["misses"] == 1 and end["hits"] - start["hits"] == 5
    assert end["leased"] == start["leased"] and end["idle"] == 1
    # an error after the lease was taken (the typed buffer is pageable host memory) returns the lease
    host = torch.zeros(size * 2, dtype=torch.uint8).pin_memory()
    with pytest.raises(tp.TpError) as e:
        tp.pack_host(torch.zeros(ex * 2, dtype=torch.uint8), 2, h, host, size * 2, 0, None, 0, tp.TP_METHOD_STAGED)
    assert e.value.code == tp.TP_ERR_BUFFER
    after = tp.resource_stats(tp.TP_RES_DEVICE)
    assert after["leased"] == start["leased"] and after["hits"] == end["hits"] + 1
    tp.resource_trim()


def test_plain_c_program_packs_and_unpacks(dev):
    # the path driven from C through the header alone (its own process, the system's HIP runtime):
    # buffers from the resource cache, data in and out through zero-copy calls, compared with
    # nested loops in C
    import subprocess
    exe = os.path.join(os.path.dirname(tp.LIB_PATH), "pack_selftest")
    assert os.path.exists(exe), "build the library first (python -m paper_2012_14363_amd.build)"
    for shape in ((), ("64", "48", "40"), ("1", "1", "1"), ("63", "47", "39"), ("16", "48", "3"), ("3", "1", "40")):
        say("pack_selftest", *shape)
        r = subprocess.run([exe, *shape], capture_output=True, text=True, timeout=120)
        assert r.returncode == 0 and r.stdout.startswith("ok"), (shape, r.stdout, r.stderr)


# ------------------------------------------------------------------ maximum sizes
def test_more_rows_than_one_launch_takes(dev):
    # 2^31 - 1 one-byte runs at stride 2: above the 2^30 rows a launch covers, so the planner splits
    # the outer dimension at its natural limit; numpy's strided slice is the reference
    n = (1 << 31) - 1
    say("max rows: generating 4 GiB")
    src = W.fills.counter_bytes_torch(91, 2 * n, dev)
    h = tp.type_from_recipe(vector(n, 1, 2, BYTE))
    out = torch.zeros(n + 1, dtype=torch.uint8, device=dev)
    say("max rows: pack")
    assert tp.pack(src, 1, h, out, n + 1, 1) == n + 1
    assert tp.last_plan().count("tile") >= 2, tp.last_plan()
    got = out.cpu().numpy()
    say("max rows: compare")
    step = 1 << 28
    for lo in range(0, n, step):          # compare in slices to bound host memory
        hi = min(n, lo + step)
        ref = W.fills.counter_bytes_numpy(91, 2 * lo, 2 * (hi - lo))[0::2]
        assert np.array_equal(got[1 + lo:1 + hi], ref), lo
    # the oracle itself on the first 2^20 runs
    ref = np.zeros(1 << 20, np.uint8)
    cc.pack(W.fills.counter_bytes_numpy(91, 0, 1 << 21), 0, 1, vector(1 << 20, 1, 2, BYTE), ref, 0)
    assert np.array_equal(got[1:1 + (1 << 20)], ref)
    say("max rows: unpack")
    back = torch.full((2 * n,), 0xA5, dtype=torch.uint8, device=dev)
    assert tp.unpack(out, n + 1, 1, back, 1, h) == n + 1
    assert torch.equal(back[0::2], out[1:]) and bool((back[1::2] == 0xA5).all())


def test_run_longer_than_one_launch_takes(dev):
    # one contiguous run of 2^31 - 1 bytes between odd addresses: fewer than the 2^30 words a launch
    # covers when they are 16 bytes wide; as byte-wide words the run is cut into pieces
    n = (1 << 31) - 1
    say("max run: generating")
    src = W.fills.counter_bytes_torch(92, n + 8, dev)
    dst = torch.zeros(n + 8, dtype=torch.uint8, device=dev)
    h = tp.type_from_recipe(contiguous(n, BYTE))
    assert tp.pack(src.data_ptr() + 1, 1, h, dst.data_ptr() + 3, n, 0) == n
    plan = tp.last_plan()
    assert plan.count("tile W=16") == 1 and "back=1 " in plan, plan
    assert torch.equal(dst[3:3 + n], src[1:1 + n])
    assert int(dst[:3].sum()) == 0 and int(dst[3 + n:].sum()) == 0
    dst.zero_()
    try:
        tp.set_override("word", 1)
        assert tp.pack(src.data_ptr() + 1, 1, h, dst.data_ptr() + 3, n, 0) == n
    finally:
        tp.set_override("word", 0)
    plan = tp.last_plan()
    assert plan.count("tile") >= 2 and "W=1 " in plan, plan
    assert torch.equal(dst[3:3 + n], src[1:1 + n])
    assert int(dst[:3].sum()) == 0 and int(dst[3 + n:].sum()) == 0
    # 16-byte words are cut as well once the limit is lowered to 2^26 words: two pieces
    dst.zero_()
    try:
        tp.set_override("max_words_per_run", 1 << 26)
        assert tp.pack(src.data_ptr() + 1, 1, h, dst.data_ptr() + 3, n, 0) == n
    finally:
        tp.set_override("max_words_per_run", 1 << 30)
    assert tp.last_plan().count("tile W=16") == 2, tp.last_plan()
    assert torch.equal(dst[3:3 + n], src[1:1 + n])
    assert int(dst[:3].sum()) == 0 and int(dst[3 + n:].sum()) == 0


def test_two_threads_two_streams(dev):
    # pack/unpack calls from different host threads on different streams may overlap
    import threading

    t = hvector(64, 1, 9000, vector(33, 24, 40, FLOAT))
    h = tp.type_from_recipe(t)
    size, ex = tp.type_size(h), tp.type_get_extent(h)[1]
    errors = []

    def worker(k):
        try:
            stream = torch.cuda.Stream()
            src_h = W.random_bytes(900 + k, ex)
            expect = np.zeros(size, np.uint8)
            cc.pack(src_h, 0, 1, t, expect, 0)
            with torch.cuda.stream(stream):
                src = to_dev(src_h, dev)
                out = torch.zeros(size, dtype=torch.uint8, device=dev)
                back = torch.full((ex,), 0xA5, dtype=torch.uint8, device=dev)
                for _ in range(50):
                    assert tp.pack(src, 1, h, out, size, 0, stream) == size
                    assert tp.unpack(out, size, 0, back, 1, h, stream) == size
                got, got_back = out.cpu().numpy(), back.cpu().numpy()
            want = np.full(ex, 0xA5, np.uint8)
            cc.unpack(expect, 0, want, 0, 1, t)
            assert np.array_equal(got, expect) and np.array_equal(got_back, want)
        except Exception as e:  # noqa: BLE001
            errors.append(e)

    say("two threads, two streams")
    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    [th.start() for th in threads]
    [th.join() for th in threads]
    assert not errors, errors[:1]
