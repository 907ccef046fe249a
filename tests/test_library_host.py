"""Host-side checks of libzcgather that need no GPU: the library loads, exports
every symbol the header declares, rejects bad arguments before touching the
GPU, and plans launches as documented."""
import ctypes
import os
import re

import numpy as np
import pytest

import subprocess

import paper_2103_03330_amd as z
from paper_2103_03330_amd import build, probe
from paper_2103_03330_amd.binding import EXPORTS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _exported_symbols(path):
    out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True)
    return {line.split()[-1] for line in out.stdout.splitlines() if " T " in line}


def test_header_and_library_agree_on_exports():
    header = open(os.path.join(ROOT, "include", "zcgather.h")).read()
    declared = set(re.findall(r"\b(zcg_[a-z0-9_]+)\s*\(", header))
    assert declared == set(EXPORTS)
    lib = z.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert z.version() == "0.2"
    # the method's library carries no measurement tooling
    exported = {s for s in _exported_symbols(build.LIB_PATH) if s.startswith("zcg")}
    assert not [s for s in exported if "measure" in s or "synthetic" in s or "probe" in s]
    assert declared <= exported


def test_probe_header_and_library_agree_on_exports():
    header = open(os.path.join(ROOT, "include", "zcg_probe.h")).read()
    declared = set(re.findall(r"\b(zcgp_[a-z0-9_]+)\s*\(", header))
    assert declared == set(probe.EXPORTS)
    lib = probe.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    exported = {s for s in _exported_symbols(build.PROBE_LIB_PATH) if s.startswith("zcg")}
    assert exported == declared
    with pytest.raises(probe.ProbeError) as e:  # argument checks come before any GPU call
        probe.measure_h2d(0)
    assert e.value.status == -1
    with pytest.raises(probe.ProbeError):
        probe.device_copy(16, 32, 24)


def test_status_strings():
    for code in range(0, -13, -1):
        assert z.strerror(code) != "unknown status"
    assert z.strerror(-99) == "unknown status"


def test_argument_checks_run_before_any_gpu_call():
    a = np.zeros((4, 4), np.float32)
    cases = [
        (lambda: z.register_table(0, 4, 4, "f32"), z.binding.EINVAL),
        (lambda: z.register_table(a, 0, 4, "f32"), z.binding.EINVAL),
        (lambda: z.register_table(a, 4, -1, "f32"), z.binding.EINVAL),
        (lambda: z.register_table(a, 4, 4, 7), z.binding.EDTYPE),
        (lambda: z.register_table(a.ctypes.data + 4, 2, 3, "f64"), z.binding.EALIGN),
        (lambda: z.register_table(a.ctypes.data + 2, 4, 3, "f32"), z.binding.EALIGN),
        (lambda: z.alloc_table(4, 4, "f32", flags=64), z.binding.EINVAL),
        (lambda: z.alloc_table(2 ** 62, 2 ** 10, "f32"), z.binding.EINVAL),
        (lambda: z.table_from_device(0, 4, 4, "f32"), z.binding.EINVAL),
        (lambda: z.table_from_device(4098, 4, 4, "f32"), z.binding.EALIGN),
        (lambda: z.pinned_alloc(-5), z.binding.EINVAL),
    ]
    for fn, want in cases:
        with pytest.raises(z.ZcgError) as e:
            fn()
        assert e.value.status == want


def test_handles_die_once():
    t = z.table_from_device(0x10000, 10, 4, "f32")
    assert t.device_ptr == 0x10000 and t.host_ptr == 0 and t.row_bytes == 16
    h = t.handle
    t.close()
    t.close()  # idempotent on the Python object
    lib = z.load_library()
    assert lib.zcg_unregister_table(h) == z.binding.EHANDLE  # the C handle is dead
    assert lib.zcg_unregister_table(None) == z.binding.EHANDLE
    assert lib.zcg_table_device_ptr(h) is None
    assert lib.zcg_gather(h, 8, 1, 16, None) == z.binding.EHANDLE


def test_gather_rejects_before_launch():
    t = z.table_from_device(0x100000, 100, 25, "f32")  # 100-byte rows at 0x100000
    lib = z.load_library()
    try:
        assert lib.zcg_gather(t.handle, None, 0, None, None) == 0  # empty list: nothing to do
        assert lib.zcg_gather(t.handle, None, 5, 0x900000, None) == z.binding.EINVAL
        assert lib.zcg_gather(t.handle, 0x800000, -1, 0x900000, None) == z.binding.EINVAL
        assert lib.zcg_gather(t.handle, 0x800004, 5, 0x900000, None) == z.binding.EALIGN
        assert lib.zcg_gather(t.handle, 0x800000, 5, 0x900002, None) == z.binding.EALIGN
        # output overlapping the table's [0x100000, 0x100000 + 10000)
        assert lib.zcg_gather(t.handle, 0x800000, 5, 0x100000 + 9996, None) == z.binding.EALIAS
        assert lib.zcg_gather(t.handle, 0x800000, 5, 0x100000 - 400, None) == z.binding.EALIAS
        # output over the index list [0x800000, +40) or over a caller's order
        assert lib.zcg_gather(t.handle, 0x800000, 5, 0x800000 + 36, None) == z.binding.EALIAS
        assert lib.zcg_gather(t.handle, 0x800000, 5, 0x800000 - 496, None) == z.binding.EALIAS
        assert lib.zcg_gather_ordered(t.handle, 0x800000, 0xA00000, 5, 0xA00000 + 32, None, None) == z.binding.EALIAS
        assert lib.zcg_gather_variant(t.handle, 0x800000, 5, 0x900000, None, 9) == z.binding.EINVAL
    finally:
        t.close()


def test_cpu_baseline_rejects_device_tables_and_bad_lists():
    t = z.table_from_device(0x100000, 100, 25, "f32")
    try:
        with pytest.raises(z.ZcgError) as e:
            z.cpu_gather_memcpy(t, np.array([1, 2]), 0x1000, 0x2000)
        assert e.value.status == z.binding.EINVAL
    finally:
        t.close()


def test_pipeline_argument_checks():
    lib = z.load_library()
    t = z.table_from_device(0x100000, 100, 25, "f32")
    out = ctypes.c_void_p()
    bufs = (ctypes.c_void_p * 2)(0x900000, 0xA00000)
    try:
        assert lib.zcg_pipeline_create(t.handle, 0, 2, bufs, None, ctypes.byref(out)) == z.binding.EINVAL
        assert lib.zcg_pipeline_create(t.handle, 10, 0, bufs, None, ctypes.byref(out)) == z.binding.EINVAL
        assert lib.zcg_pipeline_create(t.handle, 10, 17, bufs, None, ctypes.byref(out)) == z.binding.EINVAL
        assert lib.zcg_pipeline_create(t.handle, 10, 2, None, None, ctypes.byref(out)) == z.binding.EINVAL
        bad = (ctypes.c_void_p * 2)(0x900000, 0)
        assert lib.zcg_pipeline_create(t.handle, 10, 2, bad, None, ctypes.byref(out)) == z.binding.EINVAL
        odd = (ctypes.c_void_p * 2)(0x900002, 0xA00000)
        assert lib.zcg_pipeline_create(t.handle, 10, 2, odd, None, ctypes.byref(out)) == z.binding.EALIGN
        assert lib.zcg_pipeline_create(12345, 10, 2, bufs, None, ctypes.byref(out)) == z.binding.EHANDLE
        assert lib.zcg_pipeline_submit(None, None, 0, None) == z.binding.EINVAL
        assert lib.zcg_pipeline_destroy(None) == z.binding.EINVAL
    finally:
        t.close()


def plan(row_elems, dtype, table_addr=0x7F0000000000, out_addr=0x7E0000000000, n_idx=100000, **kw):
    t = z.table_from_device(table_addr, 1000, row_elems, dtype)
    try:
        return z.plan_gather(t, n_idx, out_addr, z.LaunchOpts(**kw) if kw else None)
    finally:
        t.close()


def test_plan_picks_width_group_and_variant():
    p = plan(100, "f32")  # 400-byte rows: unaligned to 128 -> ALIGNED, 16-byte lanes
    assert (p["variant"], p["vec_bytes"], p["log2_group"], p["iters"]) == (z.VARIANT_ALIGNED, 16, 5, 1)
    t = z.table_from_device(0x7F0000000000, 1000, 100, "f32")
    t_host_like = z.plan_gather(t, 1000, 0x7E0000000000, z.LaunchOpts(variant=z.VARIANT_HALFLINE))
    t.close()
    assert (t_host_like["variant"], t_host_like["log2_group"]) == (z.VARIANT_HALFLINE, 5)
    p = plan(99, "f16", variant=z.VARIANT_HALFLINE)  # 198-byte rows: 2-byte granular, wide loads
    assert (p["variant"], p["vec_bytes"], p["store_bytes"]) == (z.VARIANT_HALFLINE, 16, 2)
    p = plan(99, "f16", variant=z.VARIANT_HALFLINE, shifted_stores=2)  # 2-byte loads: no scalar path
    assert p["variant"] == z.VARIANT_ALIGNED
    p = plan(602, "f32")  # 2,408-byte rows: 8-byte lanes, a wave per row, several passes
    assert (p["variant"], p["vec_bytes"], p["store_bytes"], p["log2_group"]) == (z.VARIANT_ALIGNED, 16, 8, 6)
    assert p["iters"] == -(-(2408 + 120) // 1024)
    p = plan(602, "f32", shifted_stores=2)  # loads narrowed to the rows' own 8-byte alignment
    assert (p["vec_bytes"], p["store_bytes"], p["iters"]) == (8, 8, -(-(2408 + 120) // 512))
    p = plan(128, "f32")  # whole lines on an aligned base: no realignment needed
    assert (p["variant"], p["vec_bytes"], p["log2_group"], p["iters"]) == (z.VARIANT_ROWVEC, 16, 5, 1)
    p = plan(16, "f16")  # 32-byte rows, shorter than a line
    assert (p["variant"], p["vec_bytes"], p["log2_group"]) == (z.VARIANT_ROWVEC, 16, 1)
    p = plan(128, "f32", table_addr=0x7F0000000040)  # same rows on a base 64 bytes off the line
    assert p["variant"] == z.VARIANT_ALIGNED
    p = plan(100, "f32", table_addr=0x7F0000000004)  # base only element-aligned: shifted stores
    assert (p["vec_bytes"], p["store_bytes"]) == (16, 4)
    p = plan(100, "f32", out_addr=0x7E0000000008)
    assert (p["vec_bytes"], p["store_bytes"]) == (16, 8)
    p = plan(100, "f32", out_addr=0x7E0000000008, variant=z.VARIANT_ROWVEC)
    assert (p["vec_bytes"], p["store_bytes"]) == (8, 8)
    p = plan(3, "f16")
    assert p["vec_bytes"] == 2
    p = plan(401, "i8")  # odd byte rows: byte-granular stores under 16-byte line-aligned loads
    assert (p["variant"], p["vec_bytes"], p["store_bytes"]) == (z.VARIANT_ALIGNED, 16, 1)
    p = plan(37, "i8")
    assert (p["variant"], p["vec_bytes"]) == (z.VARIANT_ROWVEC, 1)
    p = plan(50, "f64")
    assert (p["vec_bytes"], p["store_bytes"]) == (16, 16)
    p = plan(100, "f32", variant=z.VARIANT_NAIVE)
    assert (p["variant"], p["vec_bytes"]) == (z.VARIANT_NAIVE, 4)
    p = plan(100, "f32", max_blocks=7)
    assert p["blocks"] == 7
    p = plan(100, "f32", n_idx=3)
    assert p["blocks"] == 1
    for bad in (dict(unroll=3), dict(line_bytes=48), dict(vec_bytes=2), dict(vec_bytes=3), dict(variant=5),
                dict(nt_loads=4), dict(shifted_stores=3), dict(row_splits=-1), dict(row_splits=4097), dict(half_ends=3)):
        with pytest.raises(z.ZcgError):
            plan(100, "f32", **bad)


def test_plan_splits_long_rows_of_short_lists():
    p = plan(16384, "f32", n_idx=16)  # 64 KiB rows, 16 of them: 4 passes of 4 KiB per wavefront
    assert (p["iters"] > 1, p["row_splits"], p["blocks"]) == (True, 4, 16)
    assert plan(16384, "f32", n_idx=100_000)["row_splits"] == 1  # long list: a wavefront per row
    assert plan(16384, "f32", n_idx=16, row_splits=1)["row_splits"] == 1
    assert plan(16384, "f32", n_idx=16, row_splits=4096)["row_splits"] == 16  # at least one pass each
    assert plan(602, "f32", n_idx=4)["row_splits"] == 1  # too short to be worth splitting
    assert plan(602, "f32", n_idx=4, row_splits=2, unroll=1)["row_splits"] == 2
    assert plan(100, "f32", n_idx=4, row_splits=8)["row_splits"] == 1  # one pass covers the row
    assert plan(16384, "f32", n_idx=16, variant=z.VARIANT_HALFLINE, row_splits=8)["row_splits"] == 1


def test_plan_half_line_policy():
    assert plan(100, "f32")["half_ends"] == 0  # not a half-line kernel
    assert plan(100, "f32", variant=z.VARIANT_HALFLINE)["half_ends"] == 2  # short rows: lone ends only
    assert plan(602, "f32", variant=z.VARIANT_HALFLINE)["half_ends"] == 1  # 768 bytes and more: every end
    assert plan(193, "f32", variant=z.VARIANT_HALFLINE)["half_ends"] == 1
    assert plan(191, "f32", variant=z.VARIANT_HALFLINE)["half_ends"] == 2
    assert plan(100, "f32", variant=z.VARIANT_HALFLINE, half_ends=1)["half_ends"] == 1
    assert plan(602, "f32", variant=z.VARIANT_HALFLINE, half_ends=2)["half_ends"] == 2


def covered_bytes(row_bytes, src_addr, p):
    """Replays the row kernels' lane->chunk mapping for one row on the host:
    returns the sorted list of (source byte, destination byte offset in row)."""
    w, line = p["vec_bytes"], p["line_bytes"]
    mask = (line - 1) if p["variant"] == z.VARIANT_ALIGNED else 0
    mis = src_addr & mask
    g = 1 << p["log2_group"]
    pairs = []
    for it in range(p["iters"]):
        for lane in range(g):
            off = (it * g + lane) * w - mis
            if -w < off < row_bytes:  # the chunk meets the row; bytes outside it are dropped
                assert (src_addr + off) % w == 0 or p["store_bytes"] == w
                pairs.extend((src_addr + off + b, off + b) for b in range(w)
                             if 0 <= off + b < row_bytes)
    return sorted(pairs)


@pytest.mark.parametrize("row_elems,dtype", [(100, "f32"), (602, "f32"), (120, "f32"), (257, "f16"),
                                             (1025, "f32"), (16, "f16"), (3, "f32")])
def test_lane_mapping_covers_each_row_byte_exactly_once(row_elems, dtype):
    elem = 2 if dtype == "f16" else 4
    rb = row_elems * elem
    base = 0x7F0000000000
    for variant in (z.VARIANT_ROWVEC, z.VARIANT_ALIGNED):
        for line in (64, 128):
            p = plan(row_elems, dtype, table_addr=base, variant=variant, line_bytes=line)
            for row in (0, 1, 2, 5, 77):
                src = base + row * rb
                got = covered_bytes(rb, src, p)
                assert got == [(src + b, b) for b in range(rb)]


def test_aligned_loads_touch_each_line_once(golden):
    """The paper's worked example on this kernel's mapping: the second 480-byte row
    costs 5 line requests when wave loads start on line boundaries, 8 when a
    32-lane, 4-byte-per-lane group starts at the row start."""
    rb, line = golden["example_row_bytes"], golden["example_line_bytes"]
    src = rb * golden["example_source_row"]

    def requests(mis, w, g):
        seen = set()
        n_chunks = -(-(mis + rb) // w)
        for c in range(n_chunks):
            off = c * w - mis
            if 0 <= off < rb:
                seen.add((c // g, (src + off) // line))
        return len(seen)

    assert requests(0, 4, 32) == golden["example_requests_naive"]
    assert requests(src % line, 4, 32) == golden["example_requests_shifted"]
    assert requests(src % line, 16, 64) == golden["example_requests_shifted"]


def test_handle_registry_is_thread_safe():
    """Handles are created, queried and destroyed from many threads at once."""
    import threading

    lib = z.load_library()
    errors = []

    def worker(seed):
        try:
            for i in range(300):
                t = z.table_from_device(0x100000 + 4096 * (seed * 1000 + i), 10 + i, 4, "f32")
                assert t.row_bytes == 16 and lib.zcg_table_n_rows(t.handle) == 10 + i
                p = z.plan_gather(t, 100, 0x7E0000000000)
                assert p["blocks"] >= 1
                h = t.handle
                t.close()
                assert lib.zcg_table_n_rows(h) == 0
        except Exception as e:  # noqa: BLE001
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(s,)) for s in range(8)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors[:3]


def test_pipeline_calls_reject_null_without_touching_the_gpu():
    import ctypes
    lib = z.load_library()
    slot = ctypes.c_int(-1)
    assert lib.zcg_pipeline_next(None, 0, ctypes.byref(slot)) == z.binding.EINVAL
    assert lib.zcg_pipeline_finish(None) == z.binding.EINVAL
    assert lib.zcg_pipeline_submit_wait(None, None, 0, 0, ctypes.byref(slot)) == z.binding.EINVAL
    assert lib.zcg_pipeline_release(None, 0, None) == z.binding.EINVAL
    assert lib.zcg_pipeline_destroy(None) == z.binding.EINVAL


def test_plan_says_when_a_lent_workspace_would_be_used_for_an_ordered_walk():
    """Host-resident rows of at most a line: AUTO orders a list only when it is long and dense
    enough in the table for shared link requests to outweigh the cost of building the order."""
    lib = z.load_library()

    def ordered(n_rows, dim, dtype, n_idx, parent_kind="host", **kw):
        # zcg_alloc_table needs a GPU; a view of a device table is not host-resident, so the
        # host-resident cases are planned on a handle made by hand
        t = z.table_from_device(0x7F0000000000, n_rows, dim, dtype)
        try:
            ws = z.gather_workspace_bytes(n_idx)
            o = z.LaunchOpts(workspace_dev=0x7D0000000000, workspace_bytes=ws, **kw)
            return z.plan_gather(t, n_idx, 0x7E0000000000, o)["ordered"]
        finally:
            t.close()

    # device-resident tables never order (HBM is not request-bound)
    assert ordered(10_000_000, 16, "f16", 1_000_000) == 0
    assert z.gather_workspace_bytes(0) == 0
    assert z.gather_workspace_bytes(1_000_000) >= 16_000_000
    ws = ctypes.c_int64(0)
    assert lib.zcg_gather_workspace_bytes(-1, ctypes.byref(ws)) == z.binding.EINVAL
    assert lib.zcg_gather_workspace_bytes(5, None) == z.binding.EINVAL


def test_static_order_builder_refuses_oversized_lists_before_touching_the_gpu():
    lib = z.load_library()
    assert lib.zcg_make_order_static(0x1000, z.STATIC_ORDER_MAX_IDX + 1, 100, 0x2000, None) == z.binding.ECAPACITY
    assert lib.zcg_make_order_static(0x1000, -1, 100, 0x2000, None) == z.binding.EINVAL
    assert lib.zcg_make_order_static(0x1000, 8, 0, 0x2000, None) == z.binding.EINVAL
    assert lib.zcg_make_order_static(None, 0, 100, None, None) == 0
    assert lib.zcg_make_order_static(0x1004, 8, 100, 0x2000, None) == z.binding.EALIGN


def test_order_workspace_never_shrinks_with_the_list():
    """A caller (the pipeline) sizes the order builder's workspace once for its longest list: every
    shorter list must fit, also where the builder changes its tiling (around 2^20 entries)."""
    sizes = list(range(0, 5000, 37)) + list(range((1 << 20) - 3000, (1 << 20) + 3000, 7)) + \
        [1 << 21, (1 << 21) + 1, 5_000_000, 50_000_000, (1 << 32) - 1]
    prev = -1
    for n in sorted(sizes):
        b = z.order_workspace_bytes(n)
        assert b >= prev and b % 256 == 0 and b >= 8 * n, n
        assert z.gather_workspace_bytes(n) >= b + 8 * n
        prev = b
    assert z.order_workspace_bytes(z.STATIC_ORDER_MAX_IDX) <= 9_502_720  # the static array's size


def test_a_view_dies_with_its_parent_even_if_the_handle_address_is_reused():
    """Views check the identity of their parent, not only its address: handles are heap objects,
    and the allocator readily hands a freed handle's address to the next one."""
    lib = z.load_library()
    dead_views = []
    for _ in range(200):
        parent = z.table_from_device(0x7F0000000000, 1000, 16, "f32")
        view = z.table_view(parent, 64, 10, 16, "f32")
        assert view.device_ptr == 0x7F0000000040 and view.row_bytes == 64
        nested = z.table_view(view, 64, 5, 16, "f32")  # a view of a view hangs off the same root
        assert nested.device_ptr == 0x7F0000000080
        parent.close()
        dead_views += [view, nested]
        fresh = z.table_from_device(0x7E0000000000, 1000, 16, "f32")  # may reuse the parent's address
        for v in dead_views[-2:]:
            assert lib.zcg_table_device_ptr(v.handle) is None
            assert lib.zcg_gather(v.handle, 0x1000, 1, 0x2000, None) == z.binding.EHANDLE
        fresh.close()
    for v in dead_views:
        v.close()  # a dead view can still be released, once
        assert lib.zcg_unregister_table(v.handle or 1) == z.binding.EHANDLE


def test_order_builder_refuses_overlapping_buffers():
    lib = z.load_library()
    n = 1000
    ws = z.order_workspace_bytes(n)
    idx, order, work = 0x7F0000000000, 0x7F0000100000, 0x7F0000200000
    # nothing is launched for the bad cases: the checks come first (a good call would need a GPU)
    assert lib.zcg_make_order(idx, n, 5000, idx + 4000, work, ws, None) == z.binding.EALIAS      # order over the list
    assert lib.zcg_make_order(idx, n, 5000, order, idx, ws, None) == z.binding.EALIAS            # workspace over the list
    assert lib.zcg_make_order(idx, n, 5000, work + 512, work, ws, None) == z.binding.EALIAS      # order inside the workspace
    assert lib.zcg_make_order_static(idx, n, 5000, idx + 7992, None) == z.binding.EALIAS
