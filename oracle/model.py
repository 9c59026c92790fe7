"""CPU oracle for the measured performance model.  TEST INFRASTRUCTURE ONLY.

Plain numpy/Python restatement of what the library's model must compute, for
tests; the product path never imports it.

Follows the paper's Sec. 4 (Eq. 1-3: T_device, T_oneshot, T_staged) and Sec. 6.3
(sparse measurements, pack/unpack times interpolated in two dimensions, copy
times in one).  Readings where the paper is silent:
  * the two table axes are the object size in bytes and the contiguous block
    length in bytes (the axes of the paper's pack-latency figure);
  * interpolation is bilinear on (log2 size, log2 block) of the time itself;
  * block lengths outside the measured range are clamped; sizes below it are
    clamped (latency floor); sizes above it scale the largest measured size's
    time proportionally (bandwidth regime).
"""
from __future__ import annotations

import math

import numpy as np

PRIMITIVES = ("gpu_pack", "gpu_unpack", "host_pack", "host_unpack", "d2h", "h2d")
DEVICE, ONESHOT, STAGED = 0, 1, 2


def parse(text: str) -> dict:
    """The table file: 'tp_model 1', 'sizes n ...', 'blocks m ...', then one line per primitive."""
    lines = [ln.split() for ln in text.strip().splitlines()]
    assert lines[0] == ["tp_model", "1"]
    assert lines[1][0] == "sizes" and lines[2][0] == "blocks"
    sizes = np.array([float(v) for v in lines[1][2:]])
    blocks = np.array([float(v) for v in lines[2][2:]])
    assert len(sizes) == int(lines[1][1]) and len(blocks) == int(lines[2][1])
    table = {"sizes": sizes, "blocks": blocks}
    for ln, name in zip(lines[3:], PRIMITIVES):
        assert ln[0] == name
        vals = np.array([float(v) for v in ln[1:]])
        table[name] = vals.reshape(len(sizes), len(blocks)) if name in PRIMITIVES[:4] else vals
    return table


def query(table: dict, nbytes: float, block: float) -> dict:
    """Interpolated seconds for each primitive (Sec. 6.3: pack and unpack times come from a 2D
    interpolation of sparse measurements, copy times from a 1D one).

    Written as the definition: piecewise-linear interpolation of the measured times over log2 of the
    axis values, first along the block-length axis for every measured size, then along the size axis.
    numpy.interp holds its end values outside the measured range, which is the stated clamp; beyond
    the largest measured size the time of that size grows in proportion to the bytes."""
    log_sizes, log_blocks = np.log2(table["sizes"]), np.log2(table["blocks"])
    top = float(table["sizes"][-1])
    beyond = max(1.0, nbytes / top)
    at_size, at_block = math.log2(min(nbytes, top)), math.log2(block)
    out = {}
    for name in PRIMITIVES[:4]:
        per_size = [np.interp(at_block, log_blocks, row) for row in table[name]]
        out[name] = float(np.interp(at_size, log_sizes, per_size)) * beyond
    for name in PRIMITIVES[4:]:
        out[name] = float(np.interp(at_size, log_sizes, table[name])) * beyond
    return out


def select(times: dict, t_cpu_cpu: float = 0.0, t_gpu_gpu: float = 0.0):
    """Eq. 1-3: (fastest method, [T_device, T_oneshot, T_staged])."""
    totals = [
        times["gpu_pack"] + t_gpu_gpu + times["gpu_unpack"],
        times["host_pack"] + t_cpu_cpu + times["host_unpack"],
        times["gpu_pack"] + times["d2h"] + t_cpu_cpu + times["h2d"] + times["gpu_unpack"],
    ]
    return int(np.argmin(totals)), totals
