"""Host-only properties of the launch planning (no GPU): for thousands of seeded shapes, bases,
list lengths and option sets the plan must be one the kernels can run -- enough lanes and passes
to cover the widest row span, access widths that divide what they must, a grid within its cap --
and the defaults must be the documented ones for host-resident tables."""
import numpy as np
import pytest

import paper_2103_03330_amd as z

KB = 256  # lanes per block
WAVE = 64


def check_plan(p, row_bytes, elem, table_addr, out_addr, n_idx, host, opts):
    what = (p, row_bytes, elem, hex(table_addr), hex(out_addr), n_idx, host)
    assert p["variant"] in (z.VARIANT_NAIVE, z.VARIANT_ROWVEC, z.VARIANT_ALIGNED, z.VARIANT_HALFLINE), what
    assert 1 <= p["blocks"] <= (opts.max_blocks or 65536), what
    assert p["nt_loads"] in (0, 1, 2) and p["nt_stores"] in (0, 1), what
    if p["variant"] == z.VARIANT_NAIVE:
        assert p["vec_bytes"] == elem and p["store_bytes"] == elem and p["iters"] == 1, what
        return
    w, ws, lg = p["vec_bytes"], p["store_bytes"], p["log2_group"]
    assert w in (1, 2, 4, 8, 16) and ws in (1, 2, 4, 8, 16) and elem <= w and ws <= w, what
    # stores rely on this alignment of rows and both bases
    assert row_bytes % ws == 0 and table_addr % ws == 0 and out_addr % ws == 0, what
    line_mapped = p["variant"] in (z.VARIANT_ALIGNED, z.VARIANT_HALFLINE)
    if ws < w:
        assert line_mapped, what  # only line-aligned loads may be wider than the rows' alignment
    assert p["line_bytes"] in (32, 64, 128, 256), what
    if p["variant"] == z.VARIANT_HALFLINE:
        assert p["line_bytes"] == 128 and w >= 4 and p["half_ends"] in (1, 2), what
        assert p["row_splits"] == 1, what
    else:
        assert p["half_ends"] == 0, what
    # lanes x passes cover the widest span a row can have: the row plus its distance from the
    # alignment boundary below its start
    worst = row_bytes + (p["line_bytes"] - ws if line_mapped else 0)
    assert 0 <= lg <= 6 and p["iters"] >= 1, what
    if p["iters"] == 1:
        assert (1 << lg) * w >= worst, what
    else:
        assert lg == 6, what
        assert p["iters"] * WAVE * w >= worst, what
    assert 1 <= p["row_splits"] <= 4096, what
    if p["row_splits"] > 1:
        assert p["iters"] > 1, what
        # every piece is whole passes, and the pieces cover the span
        pass_bytes = WAVE * w * p["unroll"]
        per = -(-(row_bytes + p["line_bytes"]) // p["row_splits"])
        piece = -(-per // pass_bytes) * pass_bytes
        assert piece * p["row_splits"] >= worst, what
    assert p["unroll"] in (1, 2, 4, 8), what


def test_random_plans_are_runnable():
    rng = np.random.default_rng(2103_03330)
    n = 0
    for _ in range(6000):
        elem = int(rng.choice([1, 2, 4, 8]))
        dim = int(rng.choice([1, 2, 3, 7, 16, 25, 31, 32, 33, 64, 100, 128, 129, 257, 602, 1024, 4099, 70_001]))
        row_bytes = dim * elem
        table_addr = 0x7F00_0000_0000 + int(rng.integers(0, 64)) * elem * int(rng.choice([1, 1, 16, 64]))
        out_addr = 0x7E00_0000_0000 + int(rng.integers(0, 64)) * elem
        n_idx = int(rng.choice([1, 2, 63, 1000, 2048, 4097, 110_000, 1_000_000, 50_000_000]))
        host = bool(rng.integers(0, 2))
        vec = int(rng.choice([0] + [v for v in (1, 2, 4, 8, 16) if v >= elem]))
        opts = z.LaunchOpts(variant=int(rng.integers(0, 5)), unroll=int(rng.choice([0, 1, 2, 4, 8])),
                            line_bytes=int(rng.choice([0, 32, 64, 128, 256])), vec_bytes=vec,
                            group_lanes=int(rng.choice([0, 1, 2, 16, 64])), shifted_stores=int(rng.integers(0, 3)),
                            nt_loads=int(rng.integers(0, 4)), nt_stores=int(rng.integers(0, 3)),
                            max_blocks=int(rng.choice([0, 1, 7, 300, 16384])),
                            row_splits=int(rng.choice([0, 1, 2, 5, 4096])), half_ends=int(rng.integers(0, 3)))
        p = z.plan_shape(row_bytes, elem, table_addr, out_addr, 10_000_000, n_idx, host, opts)
        check_plan(p, row_bytes, elem, table_addr, out_addr, n_idx, host, opts)
        n += 1
    assert n == 6000


def test_defaults_for_host_resident_tables():
    """What AUTO picks over the host link, on and off the line grid (the choices the GPU tests
    then run): one wavefront per row of more than a line, 8-byte lanes, half-line kernel for
    rows that are not whole lines, lone ends only below 768 bytes."""
    base, out = 0x7F00_0000_0000, 0x7E00_0000_0000

    def auto(row_bytes, elem=4, off=0, n_idx=110_000, **kw):
        return z.plan_shape(row_bytes, elem, base + off, out, 10_000_000, n_idx, True, z.LaunchOpts(**kw) if kw else None)

    p = auto(400)
    assert (p["variant"], p["vec_bytes"], p["log2_group"], p["half_ends"], p["blocks"]) == (z.VARIANT_HALFLINE, 8, 6, 2, 16384)
    p = auto(2408)
    assert (p["variant"], p["vec_bytes"], p["iters"], p["half_ends"]) == (z.VARIANT_HALFLINE, 8, 5, 1)
    assert auto(512)["variant"] == z.VARIANT_ROWVEC and auto(512)["vec_bytes"] == 8
    assert auto(512, off=64)["variant"] == z.VARIANT_HALFLINE  # whole lines, base off the line grid
    p = auto(400, off=4)  # base only element-aligned: 8-byte line-aligned loads, 4-byte stores
    assert (p["variant"], p["vec_bytes"], p["store_bytes"]) == (z.VARIANT_HALFLINE, 8, 4)
    p = auto(401, elem=1, off=3)
    assert (p["variant"], p["vec_bytes"], p["store_bytes"]) == (z.VARIANT_HALFLINE, 8, 1)
    assert auto(720)["half_ends"] == 2 and auto(768 + 16)["half_ends"] == 1
    p = auto(32, elem=2)  # a long list of rows that tile half lines: one 64-byte scalar read each
    assert (p["variant"], p["vec_bytes"], p["log2_group"]) == (z.VARIANT_HALFLINE, 16, 4)
    assert auto(32, elem=2, n_idx=20_000)["variant"] == z.VARIANT_ROWVEC
    assert auto(96)["variant"] == z.VARIANT_ROWVEC and auto(96)["log2_group"] == 4
    # a short list of long rows is split over wavefronts instead of taking the half-line kernel
    p = auto(280_004, n_idx=4)
    assert p["variant"] == z.VARIANT_ALIGNED and p["row_splits"] > 1 and p["line_bytes"] == 256
    # the same shapes out of HBM never take the half-line kernel
    for rb in (400, 2408, 512, 32):
        assert z.plan_shape(rb, 4, base, out, 10_000_000, 110_000, False)["variant"] in (z.VARIANT_ROWVEC, z.VARIANT_ALIGNED)


def test_ordered_walk_decision():
    """AUTO with lent workspace: long lists that are dense in a host-resident table of short rows."""
    base, out, ws = 0x7F00_0000_0000, 0x7E00_0000_0000, 0x7D00_0000_0000

    def ordered(row_bytes, n_rows, n_idx, host=True, **kw):
        o = z.LaunchOpts(workspace_dev=ws, workspace_bytes=z.gather_workspace_bytes(n_idx), **kw)
        return z.plan_shape(row_bytes, 2, base, out, n_rows, n_idx, host, o)["ordered"]

    assert ordered(32, 10_000_000, 1_000_000) == 1
    assert ordered(64, 10_000_000, 1_000_000) == 1
    assert ordered(128, 10_000_000, 1_000_000) == 1
    assert ordered(256, 10_000_000, 1_000_000) == 0      # longer than a line: nothing to share
    assert ordered(32, 10_000_000, 262_144) == 0          # too sparse: the build costs more than it saves
    assert ordered(32, 600_000, 200_003) == 1
    assert ordered(32, 100_000, 20_000) == 0              # too short
    assert ordered(32, 10_000_000, 1_000_000, host=False) == 0
    assert ordered(32, 10_000_000, 1_000_000, variant=z.VARIANT_ROWVEC) == 0
    o = z.LaunchOpts(workspace_dev=ws, workspace_bytes=z.gather_workspace_bytes(1_000_000) - 256)
    assert z.plan_shape(32, 2, base, out, 10_000_000, 1_000_000, True, o)["ordered"] == 0
    o = z.LaunchOpts(workspace_dev=ws + 8, workspace_bytes=z.gather_workspace_bytes(1_000_000))
    assert z.plan_shape(32, 2, base, out, 10_000_000, 1_000_000, True, o)["ordered"] == 0
    with pytest.raises(z.ZcgError):
        z.plan_shape(0, 2, base, out, 10, 10, True)
    with pytest.raises(z.ZcgError):
        z.plan_shape(32, 3, base, out, 10, 10, True)
