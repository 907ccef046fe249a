"""Host-side model of the bytes a gather moves over the host link on gfx950.

Measured behaviour (rocprofv3 counters, see the profiles): a vector load of mapped
host memory costs every 128-byte line it touches, whole; a wave-uniform load
through the scalar data cache costs one 64-byte half line. The model counts,
per row, the lines its byte range spans (and for the half-line kernel the ends
that are fetched as half lines), and the requests these make when lines of one
256-byte aligned pair travel together. The request rules rest on counters plus
time (profiles/link_request_model.txt): the link serves at most about 322-337 M
read requests per second (about 570 in flight fill it); rows of 256 bytes on and
off the 256-byte grid show identical L2-side read counts but 225 against 161 M
rows/s, the second being exactly two requests per row at the request limit. Lines shared by different rows of one list are
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


def _split(row_bytes: int, idx: np.ndarray, base_addr: int, half_ends: int):
    """Per row: lines left to vector loads (first, last, count) and which ends go through the
    scalar path. half_ends: 0 none, 1 every end that fits half a line, 2 only ends whose line
    would be requested alone (its partner in the 256-byte aligned pair is not part of the row)."""
    s, e = row_spans(row_bytes, idx, base_addr)
    first_line = s // LINE
    last_line = (e - 1) // LINE
    head = np.zeros(s.shape, dtype=bool)
    tail = np.zeros(s.shape, dtype=bool)
    vs = s.copy()
    if half_ends:
        next_line = (first_line + 1) * LINE
        head = (s % LINE) >= HALF  # the row starts in the upper half of its first line
        if half_ends == 2:
            head &= ((first_line % 2) == 1) | (e <= next_line)
        vs = np.where(head, np.minimum(e, next_line), s)
        tail = (vs < e) & (((e - 1) % LINE) < HALF)  # and ends in a lower half
        if half_ends == 2:
            tail &= ((last_line % 2) == 0) | (vs >= last_line * LINE)
    ve = np.where(tail, np.maximum(vs, last_line * LINE), e)
    return s, e, vs, ve, head, tail


def link_bytes_per_row(row_bytes: int, idx: np.ndarray, base_addr: int = 0,
                       halfline: bool = False, half_ends: int = 0) -> float:
    """Mean bytes fetched over the link per listed row (``halfline=True`` is ``half_ends=1``)."""
    half_ends = half_ends or (1 if halfline else 0)
    s, e, vs, ve, head, tail = _split(row_bytes, idx, base_addr, half_ends)
    lines = np.where(ve > vs, (ve - 1) // LINE - vs // LINE + 1, 0)
    total = lines * LINE + HALF * head.astype(np.int64) + HALF * tail.astype(np.int64)
    return float(np.mean(total))


def link_requests_per_row(row_bytes: int, idx: np.ndarray, base_addr: int = 0,
                          half_ends: int = 0) -> float:
    """Mean read requests per listed row as the link sees them: two lines of one 256-byte aligned
    pair asked for together travel as one request, a lone line is one request, a 64-byte scalar
    read is one request, and the link serves about 322-337 M requests/s whatever their size (up
    to its byte rate). The L2's own counters see lines, not pairs; the pairing is established by
    equal counters and unequal times of on-grid and off-grid rows."""
    s, e, vs, ve, head, tail = _split(row_bytes, idx, base_addr, half_ends)
    pairs = np.where(ve > vs, (ve - 1) // (2 * LINE) - vs // (2 * LINE) + 1, 0)
    return float(np.mean(pairs + head.astype(np.int64) + tail.astype(np.int64)))


NOMINAL_PCIE5_X16 = 32.0e9 * 16 * (128.0 / 130.0) / 8.0  # bytes/s on the wire, 63.0 GB/s
TLP_OVERHEAD = 24.0  # wire bytes per read completion beside its payload (framing, header, LCRC)


def link_wire_bytes_per_row(row_bytes: int, idx: np.ndarray, base_addr: int = 0, half_ends: int = 0,
                            overhead: float = TLP_OVERHEAD) -> float:
    """Mean bytes per listed row on the wire: what is fetched plus ``overhead`` bytes for every
    request's completion. Measured: consecutive memory streams at 57.6 GB/s over a link whose
    wire rate is 63.0 GB/s, i.e. 256-byte completions carry about 24 bytes each beside their
    payload; a lone 128-byte line or a 64-byte read pays the same 24 bytes for less payload. With
    this the row rates of the profiles come out within 1 %: config 2 with lone ends through
    64-byte reads, 1.5 pairs + 0.5 lines + 0.5 half lines = 540 wire bytes per row -> 116.7 M
    rows/s at 63.0 GB/s (measured 116.3); whole lines only, 572 bytes -> 110.2 M (110.1)."""
    return (link_bytes_per_row(row_bytes, idx, base_addr, half_ends=half_ends)
            + overhead * link_requests_per_row(row_bytes, idx, base_addr, half_ends))


def link_limit_rows_per_s(row_bytes: int, idx: np.ndarray, base_addr: int = 0, half_ends: int = 0,
                          wire_bytes_per_s: float = NOMINAL_PCIE5_X16, overhead: float = TLP_OVERHEAD,
                          requests_per_s: float = 322e6) -> float:
    """Rows per second the link can deliver for this request mix: the lower of the wire limit
    (wire bytes per row) and the request limit (requests per row at ~322 M/s)."""
    wire = link_wire_bytes_per_row(row_bytes, idx, base_addr, half_ends, overhead)
    reqs = link_requests_per_row(row_bytes, idx, base_addr, half_ends)
    return min(wire_bytes_per_s / wire, requests_per_s / reqs)


def useful_fraction(row_bytes: int, idx: np.ndarray, base_addr: int = 0, halfline: bool = False,
                    half_ends: int = 0) -> float:
    return row_bytes / link_bytes_per_row(row_bytes, idx, base_addr, halfline, half_ends)
