"""Seeded buffer contents.

Two kinds of fill:

* `random_bytes` / `random_grid_f64`: numpy `default_rng(seed)` draws, for
  buffers small enough to build on the host and upload.
* `counter_bytes_*`: a counter-based fill, byte i = a fixed mixing function of
  (seed, i), so a buffer of tens of GiB can be produced on the device in
  chunks while the host can still produce any slice of it without holding the
  whole thing.  The mixing function is the public splitmix64 finaliser.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK = (1 << 64) - 1


def random_bytes(seed: int, n: int) -> np.ndarray:
    """n uniform-random uint8 values from numpy's default_rng(seed)."""
    return np.random.default_rng(seed).integers(0, 256, size=int(n), dtype=np.uint8)


def random_grid_f64(seed: int, shape) -> np.ndarray:
    """float64 grid, uniform in [-1, 1)."""
    return np.random.default_rng(seed).random(size=shape, dtype=np.float64) * 2.0 - 1.0


def _mix_np(words: np.ndarray, seed: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (words + np.uint64(1)) * np.uint64(_GOLDEN) + np.uint64(seed & _MASK)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
        z = z ^ (z >> np.uint64(31))
    return z


def counter_bytes_numpy(seed: int, start: int, n: int) -> np.ndarray:
    """Bytes [start, start+n) of the counter-based stream for `seed` (uint8 array)."""
    start, n = int(start), int(n)
    if n <= 0:
        return np.zeros(0, dtype=np.uint8)
    w0, w1 = start >> 3, (start + n + 7) >> 3
    words = np.arange(w0, w1, dtype=np.uint64)
    b = _mix_np(words, seed).astype("<u8").view(np.uint8)
    off = start - (w0 << 3)
    return b[off:off + n].copy()


def counter_byte_at(seed: int, idx) -> np.ndarray:
    """Bytes of the counter-based stream at arbitrary indices (vectorised gather)."""
    idx = np.asarray(idx, dtype=np.uint64)
    z = _mix_np(idx >> np.uint64(3), seed)
    return ((z >> ((idx & np.uint64(7)) * np.uint64(8))) & np.uint64(0xFF)).astype(np.uint8)


def _s64(c: int) -> int:
    return c - (1 << 64) if c >= (1 << 63) else c


def counter_bytes_torch(seed: int, n: int, device, chunk_words: int = 1 << 24):
    """The same stream, bytes [0, n), built on `device` in chunks (torch uint8 tensor).

    int64 arithmetic wraps like uint64; logical right shifts are emulated by
    masking the sign-extension bits away.
    """
    import torch

    n = int(n)
    nwords = (n + 7) >> 3
    out = torch.empty(nwords, dtype=torch.int64, device=device)

    def lsr(x, k):
        return (x >> k) & ((1 << (64 - k)) - 1)

    for w0 in range(0, nwords, chunk_words):
        w1 = min(nwords, w0 + chunk_words)
        z = torch.arange(w0 + 1, w1 + 1, dtype=torch.int64, device=device)
        z = z * _s64(_GOLDEN) + _s64(seed & _MASK)
        z = (z ^ lsr(z, 30)) * _s64(_M1)
        z = (z ^ lsr(z, 27)) * _s64(_M2)
        z = z ^ lsr(z, 31)
        out[w0:w1] = z
    return out.view(torch.uint8)[:n]
