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
        m = re.match(r"\s+(cfg\d)\s+(\w+)\s+[\d.]+\s+[\d.]+ \([\d.]+\)\s+([\d.]+)", line)
        if m:
            out[(m.group(1), m.group(2))] = float(m.group(3))
    return out


def test_model_matches_measured_link_bytes():
    meas = measured_table()
    assert len(meas) == 8
    for k in (2, 3):
        cfg = wl.config(k)
        idx = wl.index_lists(cfg)[0]
        whole = link_model.link_bytes_per_row(cfg.row_bytes, idx)
        half = link_model.link_bytes_per_row(cfg.row_bytes, idx, halfline=True)
        # rows processed close together share a few lines, so the chip moves slightly less
        for name in ("rowvec", "aligned"):
            got = meas[(f"cfg{k}", name)]
            assert whole * 0.99 <= got <= whole * 1.001, (k, name, whole, got)
        got = meas[(f"cfg{k}", "halfline")]
        assert half * 0.99 <= got <= half * 1.001, (k, half, got)
        # the naive mapping re-requests lines straddled by two load instructions: always more
        assert meas[(f"cfg{k}", "naive")] > whole * 1.05


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
