"""Access-pattern model of the paper's indexing kernel (TEST INFRASTRUCTURE ONLY).

What Section 3.2.1 describes, stated as a map instead of a program: the kernel
runs one thread per element of the dense output, threads numbered in output
order, 32 consecutive threads forming a warp. Thread t belongs to output row
r = t div F (F = elements per row) and has position p = t mod F in it. Without
the alignment stage it copies element p of the row. With the stage, every row
is *rotated*: the thread at position p copies element (p + rot_r) mod F, where
rot_r = (first output element of row r - first source element of row r) mod 32.
Lane k of a warp then always reads a source element whose index is congruent to
k modulo 32, i.e. a warp's reads start on a line boundary of the source; the
misalignment moves to the writes. The stage applies only to rows longer than a
warp that are not a whole number of warps (the section's applicability rule).

Requests are counted as the section counts them: a warp's loads cost one link
read per distinct source line they touch.

The paper prints one worked case (a 480-byte row, the second row of the table):
8 requests without the stage, 5 with it. ``tests/golden/`` holds it.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def row_rotations(feat_size: int, idx_list: Sequence[int], shift: bool, warp_size: int = 32
                  ) -> np.ndarray:
    """rot_r for every output row (all zero when the stage is off or does not apply)."""
    src_first = np.asarray(idx_list, dtype=np.int64) * feat_size
    dst_first = np.arange(len(src_first), dtype=np.int64) * feat_size
    if not shift or feat_size <= warp_size or feat_size % warp_size == 0:
        return np.zeros_like(src_first)
    return np.mod(dst_first - src_first, warp_size)


def element_map(feat_size: int, idx_list: Sequence[int], shift: bool, warp_size: int = 32
                ) -> Tuple[np.ndarray, np.ndarray]:
    """(dst, src): for every thread, in thread order, the output element it writes and the
    source element it reads (flat element indices)."""
    src_first = np.asarray(idx_list, dtype=np.int64) * feat_size
    rot = row_rotations(feat_size, idx_list, shift, warp_size)
    t = np.arange(len(src_first) * feat_size, dtype=np.int64)
    r, p = np.divmod(t, feat_size)
    within = np.mod(p + rot[r], feat_size)  # the row's elements, rotated by rot_r
    return r * feat_size + within, src_first[r] + within


def count_read_requests(feat_size: int, idx_list: Sequence[int], shift: bool, warp_size: int = 32,
                        line_bytes: int = 128, elem_bytes: int = 4) -> int:
    """Distinct (warp, source line) pairs over all loads of one kernel pass."""
    _, src = element_map(feat_size, idx_list, shift, warp_size)
    warp = np.arange(src.size, dtype=np.int64) // warp_size
    line = (src * elem_bytes) // line_bytes
    return int(np.unique(np.stack([warp, line]), axis=1).shape[1])


def outstanding_requests(bandwidth_bytes_per_s: float, request_bytes: float, rtt_s: float) -> float:
    """Little's law sizing of Section 3.2.2: requests in flight = rate x latency."""
    return bandwidth_bytes_per_s / request_bytes * rtt_s


def gpu_share_for_requests(n_requests: float, warps_per_sm: int, n_sm: int) -> float:
    """Fraction of the GPU whose resident warps hold ``n_requests`` one-request warps."""
    return n_requests / warps_per_sm / n_sm
