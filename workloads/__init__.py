"""Seeded synthetic inputs and datatype recipes shared by the tests and the benchmark.

This package holds no part of the pack/unpack method: a *recipe* is only a
description of a nested MPI derived datatype as nested tuples, and a *fill* is
a seeded random buffer.  The CPU oracle interprets recipes by its own rules,
the HIP library is driven through its C ABI by `paper_2012_14363_amd.binding`;
neither is imported here.

Recipe grammar (mirrors the MPI constructors the paper lists in Sec. 2):

    ("named", NAME)                                   NAME in NAMED_TYPES
    ("contiguous", count, old)
    ("vector", count, blocklength, stride, old)       stride in elements of old
    ("hvector", count, blocklength, stride_bytes, old)
    ("subarray", sizes, subsizes, starts, order, old) order "C" or "F"
"""
from .recipes import (  # noqa: F401
    NAMED_TYPES,
    BYTE,
    FLOAT,
    DOUBLE,
    named,
    contiguous,
    vector,
    hvector,
    subarray,
    random_recipe,
)
from .fills import random_bytes, random_grid_f64  # noqa: F401
from . import configs  # noqa: F401
