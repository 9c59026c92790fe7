"""Datatype recipes: nested tuples naming MPI constructor calls (paper Sec. 2).

Only descriptions live here.  What a recipe *means* (its type map, size,
extent, canonical form) is computed independently by the oracle and by the
library; this module does none of that arithmetic.
"""
from __future__ import annotations

import random

# Names of the predefined types both sides know; byte sizes are each side's own business.
NAMED_TYPES = (
    "BYTE", "CHAR", "INT8", "UINT8", "INT16", "UINT16", "INT32", "UINT32",
    "INT64", "UINT64", "FLOAT", "DOUBLE",
)


def named(name: str):
    assert name in NAMED_TYPES, name
    return ("named", name)


BYTE = named("BYTE")
FLOAT = named("FLOAT")
DOUBLE = named("DOUBLE")


def contiguous(count, old):
    return ("contiguous", int(count), old)


def vector(count, blocklength, stride, old):
    return ("vector", int(count), int(blocklength), int(stride), old)


def hvector(count, blocklength, stride_bytes, old):
    return ("hvector", int(count), int(blocklength), int(stride_bytes), old)


def subarray(sizes, subsizes, starts, order, old):
    assert order in ("C", "F")
    sizes, subsizes, starts = tuple(map(int, sizes)), tuple(map(int, subsizes)), tuple(map(int, starts))
    assert len(sizes) == len(subsizes) == len(starts) >= 1
    return ("subarray", sizes, subsizes, starts, order, old)


def random_recipe(rng: random.Random, depth: int, *, max_count: int = 4,
                  allow_negative: bool = False, allow_zero: bool = False,
                  allow_overlap: bool = False, named_pool=("BYTE", "BYTE", "INT16", "FLOAT")):
    """A random small nested type for brute-force tests.

    `depth` constructor levels over a named leaf.  Unless `allow_overlap`,
    vector strides (in elements) are drawn >= blocklength so a vector never
    overlaps itself.  hvector byte strides are raw draws from a pool: this
    module does no type arithmetic, so it cannot know the child's extent, and
    an hvector may therefore describe a self-overlapping map; tests that need
    overlap-free types filter the draws with the oracle's type map.
    """
    t = named(rng.choice(named_pool))
    lo = 0 if allow_zero else 1
    for _ in range(depth):
        kind = rng.choice(("contiguous", "vector", "hvector", "subarray"))
        if kind == "contiguous":
            t = contiguous(rng.randint(lo, max_count), t)
        elif kind == "vector":
            c = rng.randint(lo, max_count)
            l = rng.randint(lo, max_count)
            if allow_overlap:
                s = rng.randint(-max_count - 2 if allow_negative else 0, max_count + 2)
            else:
                s = rng.randint(max(l, 1), max(l, 1) + 3)
                if allow_negative and rng.random() < 0.3:
                    s = -s
            t = vector(c, l, s, t)
        elif kind == "hvector":
            c = rng.randint(lo, max_count)
            l = rng.randint(lo, max_count)
            sb =rng.choice((1, 2, 3, 4, 5, 7, 8, 12, 16, 24, 32, 48, 64, 100, 128, 256, 512))
            if allow_negative and rng.random() < 0.3:
                sb = -sb
            t = hvector(c, l, sb, t)
        else:
            nd = rng.randint(1, 3)
            sizes, subs, starts = [], [], []
            for _d in range(nd):
                sz = rng.randint(1, max_count + 2)
                sub = rng.randint(lo if lo <= sz else sz, sz)
                st = rng.randint(0, sz - sub)
                sizes.append(sz), subs.append(sub), starts.append(st)
            t = subarray(sizes, subs, starts, rng.choice(("C", "F")), t)
    return t
