"""Position-weighted 64-bit checksum of an integer table — TEST INFRASTRUCTURE ONLY.

Used where a whole table is too large to keep as a fixture (the stored results
of the full-size stress configuration) or to move between devices: the table
is summarised as

    sum_i (a_i + 3) * w_i   mod 2^64,     w_i = (i * 0x9E3779B97F4A7C15 + 0x7F4A7C15) | 1,

over the flat index i of the canonical (row-major) layout.  Every weight is odd,
so changing any single cell changes the sum, and moving a value to another
position changes it unless the weights conspire.  It holds none of the
method's arithmetic.
"""
from __future__ import annotations

import numpy as np

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
OFFSET = np.uint64(0x7F4A7C15)


def table_checksum(a: np.ndarray, first_index: int = 0) -> int:
    """Checksum of `a` (any integer dtype) read row-major, its first cell having flat index `first_index`."""
    flat = np.ascontiguousarray(a).reshape(-1)
    total = np.uint64(0)
    step = 1 << 24                                    # bounded temporaries
    with np.errstate(over="ignore"):
        for lo in range(0, flat.size, step):
            x = flat[lo:lo + step].astype(np.int64).view(np.uint64) + np.uint64(3)
            i = np.arange(first_index + lo, first_index + lo + x.size, dtype=np.uint64)
            w = (i * GOLDEN + OFFSET) | np.uint64(1)
            total = total + (x * w).sum(dtype=np.uint64)
    return int(total)
