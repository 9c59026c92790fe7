"""The pins must be sharp: plant one plausible mistake at a time in a copy of the Python oracle's
constructor rules and check that the pins of tests/test_oracle_pins.py notice every one of them.
The mistakes are planted in the oracle, on the CPU; nothing here touches the library."""
import os
import types

import numpy as np
import pytest
from numpy.lib.stride_tricks import as_strided

import workloads as W
from workloads import BYTE, FLOAT, contiguous, hvector, named, subarray, vector
from oracle import typemap as py
from test_oracle_pins import TINY, _read_golden, _cuboids

INT16 = named("INT16")


def clone_oracle(placements=None, named_size=None):
    """A private copy of oracle.typemap whose `placements` (or named sizes) can be replaced."""
    src = open(py.__file__).read()
    mod = types.ModuleType("oracle_mutant")
    mod.__file__ = py.__file__
    exec(compile(src, py.__file__, "exec"), mod.__dict__)
    if placements is not None:
        original = mod.placements
        mod.placements = lambda t: placements(mod, original, t)
    if named_size is not None:
        mod.NAMED_SIZE.update(named_size)
    mod.bounds.cache_clear()
    return mod


def pin_failures(o, golden_dir):
    """Runs the core pins against oracle module `o`; returns the names of the pins that fail."""
    failed = []

    def check(name, fn):
        try:
            assert fn()
        except Exception:  # noqa: BLE001 - a mutant may also crash; that counts as noticed
            failed.append(name)

    golden = _read_golden(golden_dir)
    for name, t in TINY.items():
        size, lb, ub, blocks = golden[name]
        check("golden:" + name, lambda t=t, size=size, lb=lb, ub=ub, blocks=blocks:
              list(o.type_map(t)) == blocks and o.size(t) == size and o.bounds(t) == (lb, ub))

    def slicing(order):
        sizes, subs, starts = (5, 7, 6), (2, 4, 3), (1, 2, 3)
        raw = W.random_bytes(11, int(np.prod(sizes)) * 4)
        a = raw.view(np.float32).reshape(sizes, order=order)
        sel = a[tuple(slice(s, s + n) for s, n in zip(starts, subs))]
        expect = np.frombuffer(sel.tobytes(order=order), dtype=np.uint8)
        out = np.zeros(expect.size, dtype=np.uint8)
        o.pack(raw, 0, 1, subarray(sizes, subs, starts, order, FLOAT), out, 0)
        return np.array_equal(out, expect)

    check("numpy-slice:C", lambda: slicing("C"))
    check("numpy-slice:F", lambda: slicing("F"))

    def reshape():
        count, bl, stride = 9, 3, 5
        raw = W.random_bytes(12, count * stride * 2)
        expect = np.ascontiguousarray(raw.view(np.int16).reshape(count, stride)[:, :bl]).view(np.uint8).reshape(-1)
        out = np.zeros(expect.size, dtype=np.uint8)
        o.pack(raw, 0, 1, vector(count, bl, stride, INT16), out, 0)
        return np.array_equal(out, expect)

    check("numpy-reshape", reshape)

    def strided():
        c1, l1, sb1, c2, l2, sb2 = 3, 2, 10, 4, 2, 100
        ext_inner = (c1 - 1) * sb1 + l1 * 2
        raw = W.random_bytes(13, 1024)
        view = as_strided(raw.view(np.int16), shape=(c2, l2, c1, l1), strides=(sb2, ext_inner, sb1, 2))
        expect = np.ascontiguousarray(view).view(np.uint8).reshape(-1)
        out = np.zeros(expect.size, dtype=np.uint8)
        o.pack(raw, 0, 1, hvector(c2, l2, sb2, hvector(c1, l1, sb1, INT16)), out, 0)
        return np.array_equal(out, expect)

    check("as_strided", strided)

    def equivalents():
        e, a = (5, 3, 4), (8, 6, 5)
        raw = W.random_bytes(14, a[0] * 4 * a[1] * a[2])
        arr = raw.view(np.float32).reshape(a[2], a[1], a[0])
        expect = np.ascontiguousarray(arr[:e[2], :e[1], :e[0]]).reshape(-1).view(np.uint8)
        for t in _cuboids(e, a):
            out = np.zeros(expect.size, dtype=np.uint8)
            o.pack(raw, 0, 1, t, out, 0)
            if not np.array_equal(out, expect):
                return False
        return True

    check("paper-equivalents", equivalents)
    return failed


def test_the_unmutated_oracle_passes_every_pin(golden_dir):
    assert pin_failures(clone_oracle(), golden_dir) == []


def _vector_stride_in_bytes(mod, original, t):
    if t[0] == "vector":
        _, c, l, s, old = t
        ex = mod.extent(old)
        return (i * s + j * ex for i in range(c) for j in range(l))      # stride not scaled by the extent
    return original(t)


def _hvector_stride_in_elements(mod, original, t):
    if t[0] == "hvector":
        _, c, l, sb, old = t
        ex = mod.extent(old)
        return ((i * sb + j) * ex for i in range(c) for j in range(l))   # byte stride scaled by the extent
    return original(t)


def _contiguous_by_size(mod, original, t):
    if t[0] == "contiguous":
        _, n, old = t
        return (i * mod.size(old) for i in range(n))                      # copies packed by size, not extent
    return original(t)


def _block_elements_by_size(mod, original, t):
    if t[0] in ("vector", "hvector"):
        _, c, l, s, old = t
        ex, sz = mod.extent(old), mod.size(old)
        step = s * ex if t[0] == "vector" else s
        return (i * step + j * sz for i in range(c) for j in range(l))   # block elements packed by size
    return original(t)


def _subarray_orders_swapped(mod, original, t):
    if t[0] == "subarray":
        return original(t[:4] + ("F" if t[4] == "C" else "C",) + t[5:])
    return original(t)


def _subarray_starts_dropped(mod, original, t):
    if t[0] == "subarray":
        return original(t[:3] + (tuple(0 for _ in t[3]),) + t[4:])
    return original(t)


def _subarray_pitch_from_subsizes(mod, original, t):
    if t[0] == "subarray":
        _, sizes, subs, starts, order, old = t
        return original(("subarray", subs, subs, tuple(0 for _ in starts), order, old))
    return original(t)


def _loops_transposed(mod, original, t):
    if t[0] in ("vector", "hvector"):
        _, c, l, s, old = t
        ex = mod.extent(old)
        step = s * ex if t[0] == "vector" else s
        return (i * step + j * ex for j in range(l) for i in range(c))   # elements outer, blocks inner
    return original(t)


def _negative_stride_ignored(mod, original, t):
    if t[0] in ("vector", "hvector") and t[3] < 0:
        return original(t[:3] + (-t[3],) + t[4:])
    return original(t)


MUTANTS = {
    "vector stride taken as bytes": _vector_stride_in_bytes,
    "hvector stride taken as elements": _hvector_stride_in_elements,
    "contiguous copies placed by size instead of extent": _contiguous_by_size,
    "block elements placed by size instead of extent": _block_elements_by_size,
    "subarray C and Fortran order swapped": _subarray_orders_swapped,
    "subarray starts ignored": _subarray_starts_dropped,
    "subarray pitch from subsizes": _subarray_pitch_from_subsizes,
    "vector block and element loops transposed": _loops_transposed,
    "negative stride treated as positive": _negative_stride_ignored,
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_each_planted_mistake_is_noticed(name, golden_dir):
    failed = pin_failures(clone_oracle(placements=MUTANTS[name]), golden_dir)
    assert failed, f"no pin notices: {name}"


def test_wrong_named_sizes_and_bounds_rules_are_noticed(golden_dir):
    assert pin_failures(clone_oracle(named_size={"FLOAT": 8}), golden_dir)
    assert pin_failures(clone_oracle(named_size={"INT16": 4}), golden_dir)

    # bounds taken from the selected bytes only (ignoring a subarray's full-array span)
    mod = clone_oracle()

    def data_bounds(t):
        blocks = list(mod.type_map(t))
        if not blocks:
            return (0, 0)
        return min(d for d, _ in blocks), max(d + n for d, n in blocks)

    mod.bounds = data_bounds
    assert pin_failures(mod, golden_dir)
