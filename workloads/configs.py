"""The benchmark/parity workloads as recipes plus buffer shapes.

Shapes follow the paper's own microbenchmarks: 2D objects of 512-B pitch
described as vector or subarray (Sec. 6.2, pack figure), 64 B - 4 MiB objects
with varying contiguous block length (Sec. 6.3, pack-latency figure), the
26-neighbour radius-3 halo of 8-byte values (Sec. 6.4), and the four families
of 3D type constructions used for commit timing (Sec. 6.1, commit figure).
Everything is synthetic and seeded; only sizes and recipes are defined here.
"""
from __future__ import annotations

import itertools

from .recipes import BYTE, DOUBLE, FLOAT, contiguous, hvector, subarray, vector

SEED_BASE = 0x20121436


# ---------------------------------------------------------------- config 1
def cfg1():
    """2D vector, 64 runs of 8 B at 512-B pitch, two equivalent constructions."""
    return {
        "buffer_bytes": 32 * 1024,
        "recipes": {
            "vector": vector(64, 8, 512, BYTE),
            "hvector_of_contiguous": hvector(64, 1, 512, contiguous(8, BYTE)),
        },
        "packed_bytes": 512,
        "seed": SEED_BASE + 0,
    }


# ---------------------------------------------------------------- config 2
E0 = E1 = 512  # allocation row and plane pitch in bytes

A0_SWEEP = (1, 2, 4, 8, 16, 32, 64, 128, 256, 512)


def cfg2_point(a0: int, packed_bytes: int, a1_cap: int = 512, alloc_budget: int | None = None):
    """One point of the 3D strided-block sweep.

    The sub-block is a0 x a1 x a2 bytes inside a 512 x 512 x e2 byte
    allocation.  a1 and a2 are the most equal powers of two with
    a0*a1*a2 == packed_bytes, a1 >= a2 and a1 <= a1_cap; the outermost
    allocation dimension grows beyond 512 when a2 needs it.  With an
    `alloc_budget` (bytes) a2 is cut down to fit and the packed size shrinks.
    """
    rows = packed_bytes // a0
    assert rows * a0 == packed_bytes and rows & (rows - 1) == 0
    log_rows = rows.bit_length() - 1
    a1 = min(a1_cap, 1 << ((log_rows + 1) // 2))
    a2 = rows // a1
    if alloc_budget is not None:
        while a2 > 1 and E0 * E1 * max(512, a2) > alloc_budget:
            a2 //= 2
    e2 = max(512, a2)
    recipe = hvector(a2, 1, E0 * E1, hvector(a1, 1, E0, contiguous(a0, BYTE)))
    return {
        "a": (a0, a1, a2),
        "e": (E0, E1, e2),
        "alloc_bytes": E0 * E1 * e2,
        "packed_bytes": a0 * a1 * a2,
        "recipe": recipe,
        "seed": SEED_BASE + 1,
    }


def cfg2_sweep(packed_bytes: int, **kw):
    return [cfg2_point(a0, packed_bytes, **kw) for a0 in A0_SWEEP]


# ---------------------------------------------------------------- config 3
HALO_N = 512      # allocation edge, in grid points
HALO_R = 3        # ghost width


def _halo_range(d: int, ghost: bool, n: int, r: int):
    if d == 0:
        return (r, n - r)
    if ghost:
        return (0, r) if d < 0 else (n - r, n)
    return (r, 2 * r) if d < 0 else (n - 2 * r, n - r)


def halo_directions():
    """The 26 neighbour directions (dz, dy, dx), lexicographic, origin left out."""
    return [d for d in itertools.product((-1, 0, 1), repeat=3) if d != (0, 0, 0)]


def halo_region(direction, ghost: bool, n: int = HALO_N, r: int = HALO_R):
    """Index ranges [(z0,z1),(y0,y1),(x0,x1)] of a send (interior) or ghost region."""
    return [_halo_range(d, ghost, n, r) for d in direction]


def halo_recipe(direction, ghost: bool, n: int = HALO_N, r: int = HALO_R):
    rng = halo_region(direction, ghost, n, r)
    subs = tuple(b - a for a, b in rng)
    starts = tuple(a for a, _ in rng)
    return subarray((n, n, n), subs, starts, "C", DOUBLE)


def cfg3(n: int = HALO_N, r: int = HALO_R):
    """All 26 halo regions of an n^3 float64 grid (default 512^3) with ghost width r (default 3).

    A message packed from the send region of direction d is unpacked into the
    ghost region of direction -d (periodic self-exchange).
    """
    dirs = halo_directions()
    neg = [tuple(-c for c in d) for d in dirs]
    return {
        "grid_shape": (n, n, n),
        "directions": dirs,
        "send": [halo_recipe(d, False, n, r) for d in dirs],
        "ghost_for_send": [halo_recipe(d, True, n, r) for d in neg],
        "send_region": [halo_region(d, False, n, r) for d in dirs],
        "ghost_region_for_send": [halo_region(d, True, n, r) for d in neg],
        "seed": SEED_BASE + 2,
    }


# ---------------------------------------------------------------- config 4
CFG4_COUNT = 1 << 24
CFG4_STRIDE = 64
CFG4_BLOCKLENGTHS = (1, 2, 3, 4, 8)
CFG4_OFFSETS = tuple(range(8))


def cfg4_point(blocklength: int, count: int = CFG4_COUNT):
    return {
        "recipe": vector(count, blocklength, CFG4_STRIDE, BYTE),
        "recipe_subarray": lambda k: subarray((count, CFG4_STRIDE), (count, blocklength), (0, k), "C", BYTE),
        "source_bytes": count * CFG4_STRIDE + 64,
        "packed_bytes": count * blocklength,
        "seed": SEED_BASE + 3,
    }


# ---------------------------------------------------------------- config 5
def cfg5():
    """4-level nested type with a foldable dense innermost dimension."""
    inner = subarray((64, 64, 64), (8, 16, 64), (3, 5, 0), "C", FLOAT)
    recipe = vector(4, 1, 2, hvector(16, 1, 8192, inner))
    return {
        "recipe": recipe,
        "objects": 1000,
        "packed_bytes_per_object": 2 * 1024 * 1024,
        "seed": SEED_BASE + 4,
    }


# ------------------------------------------------- commit-timing families
def commit_recipes():
    """15 synthetic 3D type constructions in the four families of the commit figure.

    The paper's own 15 parameter sets are only in a figure; these stand in:
    a (e0, e1, e2) byte sub-block of an (a0, a1, a2) byte allocation.
    """
    shapes = [
        ((256, 512, 1024), (100, 13, 47)),
        ((512, 512, 512), (64, 64, 64)),
        ((512, 512, 512), (512, 16, 16)),
    ]
    out = []
    for (a0, a1, a2), (e0, e1, e2) in shapes:  # 0-2: subarray
        out.append(("subarray", subarray((a2, a1, a0), (e2, e1, e0), (0, 0, 0), "C", BYTE)))
    for (a0, a1, a2), (e0, e1, e2) in shapes:  # 3-5: hvector of vector
        out.append(("hvector(vector)", hvector(e2, 1, a0 * a1, vector(e1, e0, a0, BYTE))))
    for (a0, a1, a2), (e0, e1, e2) in shapes:  # 6-11: hvector of hvector of vector
        row_v = vector(1, e0, 1, BYTE)
        out.append(("hvector(hvector(vector))", hvector(e2, 1, a0 * a1, hvector(e1, 1, a0, row_v))))
        row_v4 = vector(e0 // 4, 4, 4, BYTE)
        out.append(("hvector(hvector(vector))", hvector(e2, 1, a0 * a1, hvector(e1, 1, a0, row_v4))))
    for (a0, a1, a2), (e0, e1, e2) in shapes:  # 12-14: subarray of vector
        # planes repeat at the plane type's own extent (no resized type in this grammar)
        plane = vector(e1, e0, a0, BYTE)
        out.append(("subarray(vector)", subarray((a2,), (e2,), (0,), "C", plane)))
    return out
