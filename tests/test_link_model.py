"""The link-traffic model against the rocprofv3 counter values kept under profiles/:
if the model and the measurements drift apart, the design notes are wrong."""
import os
import re

import numpy as np

import zcg_workload as wl
from paper_2103_03330_amd import link_model

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def measured_table():
    """(config, kernel) -> link bytes per row from profiles/gather_variants_cfg2_cfg3.txt."""
    out = {}
    for line in open(os.path.join(ROOT, "profiles", "gather_variants_cfg2_cfg3.txt")):
        m = re.match(r"\s+(cfg\d)\s+([\w-]+)\s+[\d.]+\s+[\d.]+ \([\d.]+\)\s+([\d.]+)\s+([\d.]+)\s+([\d.]+)", line)
        if m:
            out[(m.group(1), m.group(2))] = (float(m.group(3)), float(m.group(4)), float(m.group(5)))
    return out


def test_model_matches_measured_link_bytes():
    meas = measured_table()
    assert len(meas) == 10
    for k in (2, 3):
        cfg = wl.config(k)
        idx = wl.index_lists(cfg)[0]
        whole = link_model.link_bytes_per_row(cfg.row_bytes, idx)
        # rows processed close together share a few lines, so the chip moves slightly less
        for name in ("rowvec", "aligned"):
            got = meas[(f"cfg{k}", name)][0]
            assert whole * 0.99 <= got <= whole * 1.001, (k, name, whole, got)
        for name, policy in (("half-all", 1), ("half-lone", 2)):
            want = link_model.link_bytes_per_row(cfg.row_bytes, idx, half_ends=policy)
            got, _, reads64 = meas[(f"cfg{k}", name)]
            assert want * 0.99 <= got <= want * 1.001, (k, name, want, got)
            # the 64-byte reads the counters saw are the row ends the model sends that way
            ends = (whole - want) / 64.0
            assert abs(reads64 - ends) < 0.02, (k, name, reads64, ends)
        # the naive mapping re-requests lines straddled by two load instructions: always more
        assert meas[(f"cfg{k}", "naive")][0] > whole * 1.05
    # the default benchmark command's own counter file agrees with the lone-end policy
    text = open(os.path.join(ROOT, "profiles", "gather_cfg2_counters.txt")).read()
    per_row = float(re.search(r"^link_read_bytes_per_row = ([\d.]+)", text, re.M).group(1))
    cfg = wl.config(2)
    want = link_model.link_bytes_per_row(cfg.row_bytes, wl.index_lists(cfg)[0], half_ends=2)
    assert want * 0.99 <= per_row <= want * 1.001


def test_closed_forms():
    # 400-byte rows at 16-byte-granular offsets always span exactly four lines
    idx = np.arange(100000)
    assert link_model.link_bytes_per_row(400, idx) == 512.0
    assert link_model.link_bytes_per_row(400, idx, halfline=True) == 448.0
    # whole-line rows on an aligned base cost exactly their size; off the line grid one line more
    assert link_model.link_bytes_per_row(512, idx) == 512.0
    assert link_model.link_bytes_per_row(512, idx, base_addr=64) == 640.0
    assert link_model.link_bytes_per_row(512, idx, base_addr=64, halfline=True) == 512.0
    # rows inside one half line cost a line, or a half line through the scalar path
    assert link_model.link_bytes_per_row(32, idx) == 128.0
    assert link_model.link_bytes_per_row(32, idx, halfline=True) == 64.0
    assert abs(link_model.useful_fraction(400, idx) - 0.78125) < 1e-12
    # lone ends only: half of the 400-byte rows start on the upper line of a pair, and of those
    # half start in its upper half, half end in the lower half of a lower line -> 32 bytes saved
    assert link_model.link_bytes_per_row(400, idx, half_ends=2) == 480.0
    assert link_model.link_bytes_per_row(32, idx, half_ends=2) == 64.0  # a row inside half a line is alone
    # requests: pairs of lines, lone lines and 64-byte reads count one each
    assert link_model.link_requests_per_row(400, idx) == 2.5
    assert link_model.link_requests_per_row(400, idx, half_ends=1) == 3.0
    assert link_model.link_requests_per_row(400, idx, half_ends=2) == 2.5
    assert link_model.link_requests_per_row(512, idx) == 2.0
    assert link_model.link_requests_per_row(512, idx, base_addr=128) == 3.0
    assert link_model.link_requests_per_row(256, idx, base_addr=128) == 2.0
    assert link_model.link_requests_per_row(128, idx) == 1.0


def measured_rates():
    """label -> M rows/s from profiles/link_request_model.txt (kernel-trace times)."""
    out = {}
    for line in open(os.path.join(ROOT, "profiles", "link_request_model.txt")):
        m = re.match(r"\s{2}(\S.*?)\s{2,}([\d.]+)\s+([\d.]+)\s+([\d.]+)\s+[\d.]+\s+[\d.]+\s+[\d.]+\s+[\d.]+", line)
        if m:
            out[m.group(1).strip()] = float(m.group(3))
    return out


def test_wire_and_request_limits_explain_the_measured_row_rates():
    """Rows/s = min(wire rate / wire bytes per row, request rate / requests per row), wire bytes =
    payload + 24 per completion: within 2 % of the profiled kernels wherever the wire is the
    limit, and an upper bound within 6 % where requests are."""
    rate = measured_rates()
    cfg = wl.config(2)
    idx = wl.index_lists(cfg)[0]
    base = 0  # tables are page-aligned
    for label, policy in (("cfg2 rowvec", 0), ("cfg2 aligned", 0), ("cfg2 half-lone", 2)):
        want = link_model.link_limit_rows_per_s(cfg.row_bytes, idx, base, policy) / 1e6
        assert abs(rate[label] - want) / want < 0.02, (label, rate[label], want)
    want = link_model.link_limit_rows_per_s(cfg.row_bytes, idx, base, 1) / 1e6  # half-all: request-bound
    assert want * 0.94 < rate["cfg2 half-all"] <= want * 1.01
    uni = np.arange(0, 400_000) * 7 % 4_000_000  # any list: rows tile the grid identically
    for label, rb, off in (("rows 256 B base+0", 256, 0), ("rows 256 B base+128", 256, 128),
                           ("rows 128 B base+0", 128, 0), ("rows 512 B base+0", 512, 0)):
        want = link_model.link_limit_rows_per_s(rb, uni, off) / 1e6
        assert abs(rate[label] - want) / want < 0.02, (label, rate[label], want)
    want = link_model.link_limit_rows_per_s(512, uni, 128) / 1e6  # lone + pair + lone: both limits close
    assert want * 0.94 < rate["rows 512 B base+128"] <= want * 1.01
    # closed forms of the wire model
    assert link_model.link_wire_bytes_per_row(400, np.arange(100000), half_ends=2) == 480.0 + 24 * 2.5
    assert link_model.link_wire_bytes_per_row(256, np.arange(1000)) == 280.0
