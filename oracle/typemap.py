"""CPU oracle: MPI type-map interpreter.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition the HIP library is checked against.
Only tests, the smoke check and the benchmark's cpu_baseline leg may use it;
the product path never does, and it shares no code with the library.

What it follows: the constructor meanings the paper restates in Sec. 2
(named, contiguous, vector/hvector, subarray; from MPI-3.1 Sec. 4.1), and the
reading of MPI_Pack in Sec. 6.2: the typed buffer is "sent" into a contiguous
one.  A datatype is an *ordered* list of (byte displacement, length) blocks,
the type map; packing copies those blocks, object after object, in order.

There is no intermediate representation, no canonical form and no reordering
here, so it can be compared with the standard by eye.  Pure Python loops:
meant for types with up to ~1e6 blocks.  `oracle/typemap_c.py` wraps the same
recursion written in C for the full-size workloads.

What pins it (tests/test_oracle_pins.py, tests/test_oracle_mutations.py): the paper prints no
expected bytes, type maps or IR in its text (its figures are not part of it), so nothing here is
pinned by a value the paper states.  The pins are hand-enumerated type maps (tests/golden), closed
forms of the MPI definitions, numpy slicing / reshape / as_strided as independent readings, the
paper's lists of equivalent constructions (Sec. 2), and invariants; planted mistakes in every
constructor rule are shown to trip them.

Readings where the paper is silent (kept identical in the C twin):
  * extent = ub - lb exactly, no alignment padding;
  * a subarray has lb = 0 and ub = extent(old) * prod(sizes) whatever it selects;
  * counts of zero are legal and give an empty map; a constructor that places no
    copy of its oldtype has lb = ub = 0 (a subarray keeps its full-array extent);
  * negative strides are legal; displacements are relative to the type's origin
    (the address handed to pack/unpack), and may be negative;
  * unpack writes blocks in type-map order, so where a map overlaps itself the
    last writer wins.
"""
from __future__ import annotations

from functools import lru_cache
from math import prod

import numpy as np

NAMED_SIZE = {
    "BYTE": 1, "CHAR": 1, "INT8": 1, "UINT8": 1, "INT16": 2, "UINT16": 2,
    "INT32": 4, "UINT32": 4, "INT64": 8, "UINT64": 8, "FLOAT": 4, "DOUBLE": 8,
}


# ----------------------------------------------------------------- placements
def placements(t):
    """Displacements at which constructor `t` places copies of its oldtype, in type-map order.

    The constructor list of the paper's Sec. 2 (MPI-3.1 Sec. 4.1.2 for contiguous / vector /
    hvector, Sec. 4.1.3 for subarray), one case each."""
    kind = t[0]
    old = t[-1]
    ex = extent(old)
    if kind == "contiguous":
        _, n, _old = t
        for i in range(n):
            yield i * ex
    elif kind == "vector":
        _, c, l, s, _old = t
        for i in range(c):
            for j in range(l):
                yield (i * s + j) * ex
    elif kind == "hvector":
        _, c, l, sb, _old = t
        for i in range(c):
            for j in range(l):
                yield i * sb + j * ex
    elif kind == "subarray":
        _, sizes, subs, starts, order, _old = t
        n = len(sizes)
        # linear element index of an array position: C order makes the last
        # index the fastest, Fortran order the first.
        if order == "C":
            pitch = [prod(sizes[e + 1:]) for e in range(n)]
            loop_dims = list(range(n))            # outermost loop first
        else:
            pitch = [prod(sizes[:e]) for e in range(n)]
            loop_dims = list(range(n - 1, -1, -1))

        def rec(level, lin):
            if level == n:
                yield lin * ex
                return
            e = loop_dims[level]
            for k in range(subs[e]):
                yield from rec(level + 1, lin + (starts[e] + k) * pitch[e])

        yield from rec(0, 0)
    else:
        raise ValueError(f"unknown recipe kind {kind!r}")


# --------------------------------------------------------------------- bounds
@lru_cache(maxsize=None)  # recipes are immutable tuples; memoised only to keep nested types affordable
def bounds(t):
    """(lb, ub) of a recipe, in bytes relative to its origin (MPI-3.1 Sec. 4.1.6).

    A named type spans [0, size).  A subarray is by definition as large as the
    full array: lb = 0, ub = extent(old) * prod(sizes).  Every other
    constructor spans the union of its copies of the oldtype, each copy
    spanning the oldtype's own [lb, ub) (which, below a subarray, is wider than
    the bytes selected).  A constructor that places no copy has lb = ub = 0.
    """
    if t[0] == "named":
        return 0, NAMED_SIZE[t[1]]
    old = t[-1]
    if t[0] == "subarray":
        return 0, extent(old) * prod(t[1])
    lb_old, ub_old = bounds(old)
    spans = [(p + lb_old, p + ub_old) for p in placements(t)]
    if not spans:
        return 0, 0
    return min(a for a, _ in spans), max(b for _, b in spans)


def extent(t) -> int:
    lb, ub = bounds(t)
    return ub - lb


def size(t) -> int:
    """Number of data bytes in one object: the sum of block lengths."""
    return sum(n for _, n in type_map(t))


# ------------------------------------------------------------------- type map
def type_map(t, d: int = 0):
    """Yield the (displacement, length) blocks of recipe `t` placed at displacement d: the MPI
    type map (MPI-3.1 Sec. 4.1), which Sec. 2 of the paper takes as the meaning of a datatype."""
    if t[0] == "named":
        yield (d, NAMED_SIZE[t[1]])
        return
    old = t[-1]
    for p in placements(t):
        yield from type_map(old, d + p)


def byte_displacements(t, incount: int = 1):
    """Every selected byte's displacement, in packed order, for `incount` objects."""
    ex = extent(t)
    out = []
    for obj in range(incount):
        for d, n in type_map(t, obj * ex):
            out.extend(range(d, d + n))
    return out


def has_overlap(t, incount: int = 1) -> bool:
    """True if some byte is selected more than once by `incount` objects of `t` (MPI-3.1 Sec. 4.1:
    such a type may be sent from but not received into; the tests use this to decide whether an
    unpack has a unique result).  Pinned in tests/test_oracle_pins.py by hand-worked cases."""
    b = byte_displacements(t, incount)
    return len(set(b)) != len(b)


# ---------------------------------------------------------------- pack/unpack
def pack(inbuf: np.ndarray, origin: int, incount: int, t, outbuf: np.ndarray, position: int) -> int:
    """MPI_Pack (paper Sec. 6.2: the typed buffer is sent into a contiguous one): copy `incount` objects of type `t` whose origin is inbuf[origin]
    to outbuf[position:], returning the new position.  Raises if it would not fit."""
    ex = extent(t)
    if position + incount * size(t) > outbuf.size:
        raise ValueError("truncate")
    p = position
    for obj in range(incount):
        for d, n in type_map(t, origin + obj * ex):
            if d < 0 or d + n > inbuf.size:
                raise IndexError("type map leaves the buffer")
            outbuf[p:p + n] = inbuf[d:d + n]
            p += n
    return p


def unpack(inbuf: np.ndarray, position: int, outbuf: np.ndarray, origin: int, outcount: int, t) -> int:
    """MPI_Unpack: the mirror of `pack`; blocks are written in type-map order."""
    ex = extent(t)
    if position + outcount * size(t) > inbuf.size:
        raise ValueError("truncate")
    p = position
    for obj in range(outcount):
        for d, n in type_map(t, origin + obj * ex):
            if d < 0 or d + n > outbuf.size:
                raise IndexError("type map leaves the buffer")
            outbuf[d:d + n] = inbuf[p:p + n]
            p += n
    return p
