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


def _segment(axis, x):
    """(index i, weight w): x sits at (1-w)*axis[i] + w*axis[i+1] on a log2 scale, clamped."""
    if len(axis) == 1 or x <= axis[0]:
        return 0, 0.0
    if x >= axis[-1]:
        return len(axis) - 2, 1.0
    i = 0
    while x > axis[i + 1]:
        i += 1
    return i, (math.log2(x) - math.log2(axis[i])) / (math.log2(axis[i + 1]) - math.log2(axis[i]))


def query(table: dict, nbytes: float, block: float) -> dict:
    """Interpolated seconds for each primitive."""
    sizes, blocks = table["sizes"], table["blocks"]
    scale = nbytes / sizes[-1] if nbytes > sizes[-1] else 1.0
    si, sw = _segment(sizes, min(nbytes, sizes[-1]))
    bi, bw = _segment(blocks, block)
    s1, b1 = min(si + 1, len(sizes) - 1), min(bi + 1, len(blocks) - 1)
    out = {}
    for name in PRIMITIVES[:4]:
        g = table[name]
        lo = (1 - bw) * g[si, bi] + bw * g[si, b1]
        hi = (1 - bw) * g[s1, bi] + bw * g[s1, b1]
        out[name] = ((1 - sw) * lo + sw * hi) * scale
    for name in PRIMITIVES[4:]:
        v = table[name]
        out[name] = ((1 - sw) * v[si] + sw * v[s1]) * scale
    return out


def select(times: dict, t_cpu_cpu: float = 0.0, t_gpu_gpu: float = 0.0):
    """Eq. 1-3: (fastest method, [T_device, T_oneshot, T_staged])."""
    totals = [
        times["gpu_pack"] + t_gpu_gpu + times["gpu_unpack"],
        times["host_pack"] + t_cpu_cpu + times["host_unpack"],
        times["gpu_pack"] + times["d2h"] + t_cpu_cpu + times["h2d"] + times["gpu_unpack"],
    ]
    return int(np.argmin(totals)), totals
