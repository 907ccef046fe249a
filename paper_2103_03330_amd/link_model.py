"""Host-side model of the bytes a gather moves over the host link on gfx950.

Measured behaviour (rocprofv3 counters, see the profiles): a vector load of mapped
host memory costs every 128-byte line it touches, whole; a wave-uniform load
through the scalar data cache costs one 64-byte half line. The model counts,
per row, the lines its byte range spans (and for the half-line kernel the ends
that are fetched as half lines). Lines shared by different rows of one list are
counted once per row: the hardware saves a little more when such rows are
processed close together.
"""
from __future__ import annotations

import numpy as np

LINE = 128
HALF = 64


def row_spans(row_bytes: int, idx: np.ndarray, base_addr: int = 0):
    """Start and end byte address of every listed row."""
    start = base_addr + np.asarray(idx, dtype=np.int64) * row_bytes
    return start, start + row_bytes


def link_bytes_per_row(row_bytes: int, idx: np.ndarray, base_addr: int = 0,
                       halfline: bool = False) -> float:
    """Mean bytes fetched over the link per listed row."""
    s, e = row_spans(row_bytes, idx, base_addr)
    first_line = s // LINE
    last_line = (e - 1) // LINE
    lines = last_line - first_line + 1
    total = lines * LINE
    if halfline:
        head = (s % LINE) >= HALF  # the row starts in the upper half of its first line
        after_head = np.where(head, np.minimum(e, (first_line + 1) * LINE), s)
        tail = (after_head < e) & (((e - 1) % LINE) < HALF)  # and ends in a lower half
        total = total - HALF * head.astype(np.int64) - HALF * tail.astype(np.int64)
    return float(np.mean(total))


def useful_fraction(row_bytes: int, idx: np.ndarray, base_addr: int = 0, halfline: bool = False) -> float:
    return row_bytes / link_bytes_per_row(row_bytes, idx, base_addr, halfline)
