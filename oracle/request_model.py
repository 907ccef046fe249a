"""Access-pattern model of the paper's indexing kernel (TEST INFRASTRUCTURE ONLY).

Follows the steps of the indexing kernel of Section 3.2.1 (Listing 2) in the
paper's notation -- one thread per linear element ``i``, ``dstIdx = i / feat_size``,
``offset = i % feat_size``, and, when enabled, the circular-shift stage that
rotates each row's thread->element mapping by ``diff`` -- and counts the link
read requests the way the section counts them: one request per distinct
(warp, cache line) pair touched by a warp's loads.

The paper prints one worked case (a 480-byte row, second row of the table):
8 requests without the shift, 5 with it. ``tests/golden/`` holds it.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def thread_offsets(i: int, feat_size: int, idx_list: Sequence[int], shift: bool,
                   warp_size: int = 32) -> Tuple[int, int]:
    """(dstOffset, srcOffset), in elements, handled by the thread with linear index ``i``."""
    dstIdx = i // feat_size
    offset = i % feat_size
    dstStart = dstIdx * feat_size
    srcStart = idx_list[dstIdx] * feat_size
    dstOffset = offset + dstStart
    srcOffset = offset + srcStart
    # Applicability rule: rows shorter than a line, or a whole number of lines, are left alone.
    if shift and feat_size > warp_size and feat_size % warp_size != 0:
        diff = (dstStart - srcStart) % warp_size  # Python's % is already non-negative
        dstOffset += diff
        srcOffset += diff
        if srcOffset >= srcStart + feat_size:  # wrapped past the row end: rotate back
            dstOffset -= feat_size
            srcOffset -= feat_size
    return dstOffset, srcOffset


def copy_pairs(feat_size: int, idx_list: Sequence[int], shift: bool, warp_size: int = 32
               ) -> List[Tuple[int, int]]:
    """All (dstOffset, srcOffset) pairs the kernel performs for this index list."""
    n = len(idx_list) * feat_size
    return [thread_offsets(i, feat_size, idx_list, shift, warp_size) for i in range(n)]


def count_read_requests(feat_size: int, idx_list: Sequence[int], shift: bool, warp_size: int = 32,
                        line_bytes: int = 128, elem_bytes: int = 4) -> int:
    """Distinct (warp, source cache line) pairs over all loads of one kernel pass."""
    seen = set()
    n = len(idx_list) * feat_size
    for i in range(n):
        _, srcOffset = thread_offsets(i, feat_size, idx_list, shift, warp_size)
        seen.add((i // warp_size, (srcOffset * elem_bytes) // line_bytes))
    return len(seen)


def outstanding_requests(bandwidth_bytes_per_s: float, request_bytes: float, rtt_s: float) -> float:
    """Little's law sizing of Section 3.2.2: requests in flight = rate x latency."""
    return bandwidth_bytes_per_s / request_bytes * rtt_s


def gpu_share_for_requests(n_requests: float, warps_per_sm: int, n_sm: int) -> float:
    """Fraction of the GPU whose resident warps hold ``n_requests`` one-request warps."""
    return n_requests / warps_per_sm / n_sm
