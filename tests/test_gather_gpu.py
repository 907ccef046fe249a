"""GPU parity: the HIP gather, called through the C ABI, against the CPU oracle,
bit for bit, on the same seeded inputs. Integer/byte work: the bar is exact."""
import numpy as np
import pytest

import zcg_workload as wl
from oracle import gather as oracle_gather

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
z = pytest.importorskip("paper_2103_03330_amd")
from paper_2103_03330_amd import probe  # noqa: E402

ALL_VARIANTS = [z.VARIANT_AUTO, z.VARIANT_NAIVE, z.VARIANT_ROWVEC, z.VARIANT_ALIGNED,
                z.VARIANT_HALFLINE]
TORCH_DT = {"f16": torch.float16, "f32": torch.float32, "i8": torch.int8, "f64": torch.float64}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    z.load_library()
    torch.cuda.set_device(0)


def host_table(n_rows, dim, dtype, seed, mode=wl.FILL_UNIFORM, flags=z.ALLOC_DEFAULT):
    t = z.alloc_table(n_rows, dim, dtype, flags)
    wl.fill_table_ptr(t.host_ptr, n_rows, dim, dtype, seed, mode)
    return t


def run_gather(table, idx_np, dtype, opts=None, out=None):
    idx_dev = torch.from_numpy(np.ascontiguousarray(idx_np, dtype=np.int64)).cuda()
    if out is None:
        out = torch.full((len(idx_np), table.dim), -7, dtype=TORCH_DT[dtype], device="cuda")
    z.gather_ex(table, idx_dev, out, opts, n_idx=len(idx_np))
    torch.cuda.synchronize()
    return out


def assert_same_bits(got_torch, want_np, what=""):
    got = got_torch.cpu().numpy()
    assert got.shape == want_np.shape, what
    if got.tobytes() != want_np.tobytes():
        bad = np.argwhere(got.view(np.uint8).reshape(got.shape[0], -1)
                          != want_np.view(np.uint8).reshape(got.shape[0], -1))
        raise AssertionError(f"{what}: {len(bad)} bytes differ, first at row/byte {bad[0]}")


SHAPES = [
    # (n_rows, dim, dtype): row bytes 400, 2408, 512, 64, 4, 12, 28, 2, 514, 2048, 4100, 6
    (5000, 100, "f32"), (3000, 602, "f32"), (4096, 128, "f32"), (9000, 16, "f32"),
    (777, 1, "f32"), (1001, 3, "f32"), (1500, 7, "f32"), (513, 1, "f16"), (2000, 257, "f16"),
    (1200, 1024, "f16"), (900, 1025, "f32"), (1100, 3, "f16"),
    # rows inside one half line (32 B, 64 B), straddling halves (48 B, 80 B, 200 B), 2-byte odd
    (4000, 16, "f16"), (4000, 16, "f32"), (3000, 12, "f32"), (3000, 20, "f32"), (2500, 50, "f32"),
    (2500, 98, "f16"), (1300, 99, "f16"), (700, 1023, "f32"),
    # 1-byte (int8 / fp8) and 8-byte elements: odd byte rows, sub-line, long, line multiples
    (3000, 1, "i8"), (3000, 37, "i8"), (2500, 100, "i8"), (2000, 401, "i8"), (900, 2049, "i8"),
    (2000, 512, "i8"), (1500, 1, "f64"), (1500, 50, "f64"), (800, 301, "f64"),
    # the row sizes of the alignment experiment (Section 4.2): 1024 ... 1044 bytes
    (1500, 256, "f32"), (1500, 257, "f32"), (1500, 258, "f32"), (1500, 259, "f32"), (1500, 260, "f32"),
    (1500, 261, "f32"),
]


@pytest.mark.parametrize("n_rows,dim,dtype", SHAPES)
def test_all_variants_match_oracle(n_rows, dim, dtype):
    table = host_table(n_rows, dim, dtype, seed=n_rows + dim)
    try:
        host = table.host_array()
        for n_idx in (1, 63, 4099):
            idx = wl.uniform_indices(n_idx, n_rows, seed=n_idx)
            want = oracle_gather(host, idx)
            for variant in ALL_VARIANTS:
                got = run_gather(table, idx, dtype, z.LaunchOpts(variant=variant))
                assert_same_bits(got, want, f"{dtype} dim={dim} n_idx={n_idx} variant={variant}")
    finally:
        table.close()


@pytest.mark.parametrize("dim,dtype", [(100, "f32"), (602, "f32"), (257, "f16"), (2050, "f16"),
                                       (401, "i8"), (301, "f64")])
def test_launch_knobs_do_not_change_the_result(dim, dtype):
    n_rows = 3001
    table = host_table(n_rows, dim, dtype, seed=dim)
    try:
        idx = wl.uniform_indices(10007, n_rows, seed=3)
        want = oracle_gather(table.host_array(), idx)
        for variant in (z.VARIANT_ROWVEC, z.VARIANT_ALIGNED, z.VARIANT_HALFLINE):
            for unroll in (1, 2, 4, 8):
                for line in (32, 64, 128, 256):
                    o = z.LaunchOpts(variant=variant, unroll=unroll, line_bytes=line)
                    assert_same_bits(run_gather(table, idx, dtype, o), want, f"u{unroll} l{line}")
            for vec in (1, 2, 4, 8, 16):
                if vec < table.elem_bytes:
                    continue
                o = z.LaunchOpts(variant=variant, vec_bytes=vec, nt_loads=1, nt_stores=2)
                assert_same_bits(run_gather(table, idx, dtype, o), want, f"vec{vec}")
            for vec in (8, 16):  # narrow loads instead of shifted stores
                if vec < table.elem_bytes:
                    continue
                o = z.LaunchOpts(variant=variant, vec_bytes=vec, shifted_stores=2, group_lanes=16)
                assert_same_bits(run_gather(table, idx, dtype, o), want, f"noshift vec{vec}")
            # one block only: the grid-stride loop does all the work
            o = z.LaunchOpts(variant=variant, max_blocks=1)
            assert_same_bits(run_gather(table, idx, dtype, o), want, "max_blocks=1")
            for half_ends in (1, 2):  # which row ends the half-line kernel takes through 64-byte reads
                for unroll in (1, 4):
                    o = z.LaunchOpts(variant=variant, half_ends=half_ends, unroll=unroll, max_blocks=64)
                    assert_same_bits(run_gather(table, idx, dtype, o), want, f"half_ends{half_ends} u{unroll}")
            # several wavefronts per row (rows wider than one wave pass; else the knob is moot)
            for splits, unroll, vec in ((2, 1, 0), (3, 2, 0), (7, 1, 4), (64, 1, 2), (4096, 1, 1)):
                if vec and vec < table.elem_bytes:
                    continue
                o = z.LaunchOpts(variant=variant, row_splits=splits, unroll=unroll, vec_bytes=vec,
                                 max_blocks=0 if splits != 3 else 5)
                assert_same_bits(run_gather(table, idx, dtype, o), want, f"splits{splits} u{unroll} v{vec}")
        o = z.LaunchOpts(variant=z.VARIANT_NAIVE, max_blocks=3, nt_loads=1)
        assert_same_bits(run_gather(table, idx, dtype, o), want, "naive 3 blocks")
    finally:
        table.close()


def test_raw_bit_patterns_and_invariants():
    n_rows, dim = 2048, 100
    table = host_table(n_rows, dim, "f32", seed=8, mode=wl.FILL_RAW_BITS)
    try:
        host = table.host_array()
        # identity list reproduces the table, NaN payloads included
        got = run_gather(table, np.arange(n_rows), "f32")
        assert got.cpu().numpy().tobytes() == host.tobytes()
        # duplicates give identical rows; permutation of the list permutes the rows
        idx = wl.uniform_indices(5000, n_rows, seed=1)
        perm = np.random.default_rng(0).permutation(5000)
        a = run_gather(table, idx, "f32").cpu().numpy().view(np.uint32)
        b = run_gather(table, idx[perm], "f32").cpu().numpy().view(np.uint32)
        assert (a[perm] == b).all()
        assert a.tobytes() == oracle_gather(host, idx).tobytes()
    finally:
        table.close()


def test_empty_list_and_argument_errors():
    table = host_table(100, 8, "f32", seed=1)
    try:
        out = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
        idx = torch.zeros(4, dtype=torch.int64, device="cuda")
        z.gather(table, idx, out, n_idx=0)  # no launch, no error
        with pytest.raises(z.ZcgError) as e:
            z.gather(table, idx, out, n_idx=-1)
        assert e.value.status == -1
        with pytest.raises(z.ZcgError) as e:  # output inside the table
            z.gather(table, idx, table.device_ptr + 64, n_idx=4)
        assert e.value.status == -7
        with pytest.raises(z.ZcgError) as e:  # output not aligned to the element
            z.gather(table, idx, out.data_ptr() + 2, n_idx=2)
        assert e.value.status == -6
        with pytest.raises(z.ZcgError) as e:
            z.gather_ex(table, idx, out, z.LaunchOpts(unroll=3), n_idx=4)
        assert e.value.status == -1
        with pytest.raises(TypeError):
            z.gather(table, idx.to(torch.int32), out)
        assert z.validate_indices(table, idx) == 0
        bad = torch.tensor([0, 100, -1, 99, 1 << 40], dtype=torch.int64, device="cuda")
        assert z.validate_indices(table, bad) == 3
    finally:
        table.close()
    with pytest.raises(z.ZcgError) as e:  # dead handle
        z.gather(table.__class__(12345, 100, 8, z.F32), idx, out, n_idx=4)
    assert e.value.status == -3


@pytest.mark.parametrize("byte_off", [4, 8, 16, 48, 100])
def test_unaligned_bases(byte_off):
    """Table base and output base off the 16 B / line grid: the kernels must pick
    their access width and alignment from the real addresses."""
    n_rows, dim = 2000, 100
    table = host_table(n_rows + 1, dim, "f32", seed=5)
    try:
        host = table.host_array().reshape(-1)
        sub = host[byte_off // 4: byte_off // 4 + n_rows * dim].reshape(n_rows, dim)
        view = z.table_from_device(table.device_ptr + byte_off, n_rows, dim, "f32")
        idx = wl.uniform_indices(3000, n_rows, seed=2)
        want = oracle_gather(np.ascontiguousarray(sub), idx)
        for variant in ALL_VARIANTS:
            got = run_gather(view, idx, "f32", z.LaunchOpts(variant=variant))
            assert_same_bits(got, want, f"table+{byte_off} variant={variant}")
            # output base shifted as well
            buf = torch.zeros(3000 * dim + 64, dtype=torch.float32, device="cuda")
            o = buf[byte_off // 4: byte_off // 4 + 3000 * dim].view(3000, dim)
            got = run_gather(view, idx, "f32", z.LaunchOpts(variant=variant), out=o)
            assert_same_bits(got, want, f"out+{byte_off} variant={variant}")
            assert float(buf[: byte_off // 4].abs().sum()) == 0.0  # nothing written before out
            assert float(buf[byte_off // 4 + 3000 * dim:].abs().sum()) == 0.0  # nor after
        view.close()
    finally:
        table.close()


@pytest.mark.parametrize("dim", [100, 257, 602, 128, 16])
def test_auto_on_host_resident_views_off_the_line_grid(dim):
    """A table that starts anywhere inside a pinned allocation (zcg_table_view keeps it
    host-resident): the default call must plan from the real address -- half-line kernel with
    shifted stores for rows longer than a line -- and still be exact."""
    n_rows, n_idx = 2000, 3000
    parent = host_table(n_rows + 2, dim, "f32", seed=dim + 1)
    try:
        flat = parent.host_array().reshape(-1)
        idx = wl.uniform_indices(n_idx, n_rows, seed=2)
        idx[:2] = (0, n_rows - 1)
        for byte_off in (4, 8, 16, 48, 64, 100, 128, 4 * dim):
            view = z.table_view(parent, byte_off, n_rows, dim, "f32")
            assert view.device_ptr == parent.device_ptr + byte_off
            assert view.host_ptr == parent.host_ptr + byte_off
            sub = np.ascontiguousarray(flat[byte_off // 4: byte_off // 4 + n_rows * dim].reshape(n_rows, dim))
            want = oracle_gather(sub, idx)
            buf = torch.zeros(n_idx * dim + 64, dtype=torch.float32, device="cuda")
            for out_off in (0, byte_off % 64):
                out = buf[out_off // 4: out_off // 4 + n_idx * dim].view(n_idx, dim)
                plan = z.plan_gather(view, n_idx, out)
                if dim * 4 > 128 and (dim * 4) % 128:
                    assert plan["variant"] == z.VARIANT_HALFLINE, (byte_off, plan)
                    if byte_off % 8 or out_off % 8:
                        assert plan["store_bytes"] < plan["vec_bytes"], (byte_off, plan)  # shifted stores
                if dim == 128:  # whole-line rows: realigned only when the base is off the line grid
                    want_variant = z.VARIANT_ROWVEC if byte_off % 128 == 0 else z.VARIANT_HALFLINE
                    assert plan["variant"] == want_variant, (byte_off, plan)
                buf.zero_()
                got = run_gather(view, idx, "f32", None, out=out)
                assert_same_bits(got, want, f"view+{byte_off} out+{out_off} dim={dim} plan={plan}")
                assert not bool(buf[: out_off // 4].view(torch.int32).any())
                assert not bool(buf[out_off // 4 + n_idx * dim:].view(torch.int32).any())
            # the DMA baseline reads through the view's host address
            staging = z.pinned_alloc(n_idx * dim * 4)
            out = torch.zeros((n_idx, dim), dtype=torch.float32, device="cuda")
            z.cpu_gather_memcpy(view, idx, staging, out, n_threads=2)
            torch.cuda.synchronize()
            assert_same_bits(out, want, f"cpu baseline on view+{byte_off}")
            z.pinned_free(staging)
            view.close()
        with pytest.raises(z.ZcgError) as e:  # past the parent's end
            z.table_view(parent, 8, n_rows + 2, dim, "f32")
        assert e.value.status == -1
        with pytest.raises(z.ZcgError) as e:
            z.table_view(parent, 2, n_rows, dim, "f32")
        assert e.value.status == -6
        view = z.table_view(parent, 16, n_rows, dim, "f32")
    finally:
        parent.close()
    # the parent is gone: the view is dead for every call, and can still be released
    idx_dev = torch.zeros(4, dtype=torch.int64, device="cuda")
    out = torch.zeros((4, dim), dtype=torch.float32, device="cuda")
    with pytest.raises(z.ZcgError) as e:
        z.gather(view, idx_dev, out)
    assert e.value.status == -3
    view.close()


_KEPT_ALIVE = []  # see test_uncached_host_table


def test_uncached_host_table():
    """ZCG_ALLOC_UNCACHED (extended fine-grained host memory). The table is kept until the
    process ends on purpose: memory of this kind is not handed back while the GPU may still
    hold lines of it."""
    n_rows, dim = 3000, 100
    table = host_table(n_rows, dim, "f32", seed=77, flags=z.ALLOC_UNCACHED)
    _KEPT_ALIVE.append(table)
    idx = wl.uniform_indices(5000, n_rows, seed=4)
    want = oracle_gather(table.host_array(), idx)
    for variant in ALL_VARIANTS:
        assert_same_bits(run_gather(table, idx, "f32", z.LaunchOpts(variant=variant)), want, "uncached")


def test_hbm_resident_table_and_noncoherent_host_table():
    n_rows, dim = 6000, 602
    np_table = wl.make_table(n_rows, dim, "f32", seed=21)
    idx = wl.uniform_indices(7001, n_rows, seed=6)
    want = oracle_gather(np_table, idx)
    dev = torch.from_numpy(np_table).cuda()
    t = z.table_from_device(dev, n_rows, dim, "f32")
    for variant in ALL_VARIANTS:
        assert_same_bits(run_gather(t, idx, "f32", z.LaunchOpts(variant=variant)), want, "hbm")
    t.close()
    # a short list of long rows out of HBM: the rows are shared among wavefronts
    wide = wl.make_table(30, 50_001, "f32", seed=22)
    dev_wide = torch.from_numpy(wide).cuda()
    t = z.table_from_device(dev_wide, 30, 50_001, "f32")
    short = np.array([29, 0, 7, 29], np.int64)
    probe = torch.zeros((4, 50_001), dtype=torch.float32, device="cuda")
    assert z.plan_gather(t, 4, probe)["row_splits"] > 1
    for variant in ALL_VARIANTS:
        assert_same_bits(run_gather(t, short, "f32", z.LaunchOpts(variant=variant)),
                         oracle_gather(wide, short), "hbm wide")
    t.close()
    t = host_table(n_rows, dim, "f32", seed=21, flags=z.ALLOC_NONCOHERENT)
    for variant in ALL_VARIANTS:
        assert_same_bits(run_gather(t, idx, "f32", z.LaunchOpts(variant=variant)), want, "noncoh")
    t.close()


def test_cpu_gather_memcpy_baseline_matches_oracle():
    n_rows, dim = 20000, 100
    table = host_table(n_rows, dim, "f32", seed=4)
    try:
        idx = wl.uniform_indices(30011, n_rows, seed=9)
        want = oracle_gather(table.host_array(), idx)
        n_bytes = idx.size * table.row_bytes
        staging = z.pinned_alloc(n_bytes)
        for chunk in (0, 4096, 50000):
            out = torch.zeros((idx.size, dim), dtype=torch.float32, device="cuda")
            if chunk:
                z.cpu_gather_memcpy_chunked(table, idx, staging, out, chunk, n_threads=4)
            else:
                z.cpu_gather_memcpy(table, idx, staging, out, n_threads=4)
            torch.cuda.synchronize()
            assert_same_bits(out, want, f"cpu baseline chunk={chunk}")
        with pytest.raises(z.ZcgError) as e:
            z.cpu_gather_memcpy(table, np.array([0, n_rows]), staging, out)
        assert e.value.status == -8
        z.pinned_free(staging)
    finally:
        table.close()


def test_gather_on_a_side_stream():
    n_rows, dim = 5000, 100
    table = host_table(n_rows, dim, "f32", seed=2)
    try:
        idx = wl.uniform_indices(20000, n_rows, seed=1)
        want = oracle_gather(table.host_array(), idx)
        idx_dev = torch.from_numpy(idx).cuda()
        out = torch.zeros((idx.size, dim), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        s = torch.cuda.Stream()
        z.gather(table, idx_dev, out, stream=s)
        s.synchronize()
        assert_same_bits(out, want, "side stream")
    finally:
        table.close()


def test_gather_on_a_cu_masked_stream():
    """Resource provisioning: a stream bound to a few compute units still gathers correctly."""
    n_rows, dim = 5000, 100
    table = host_table(n_rows, dim, "f32", seed=12)
    try:
        idx = wl.uniform_indices(30000, n_rows, seed=5)
        want = oracle_gather(table.host_array(), idx)
        idx_dev = torch.from_numpy(idx).cuda()
        n_cus = z.device_cu_count(0)
        assert n_cus >= 8
        for cus in (list(range(8)), list(range(40)), list(range(8, n_cus)), list(range(n_cus))):
            ms = z.stream_create_cu_mask(cus)
            out = torch.zeros((idx.size, dim), dtype=torch.float32, device="cuda")
            torch.cuda.synchronize()
            z.gather(table, idx_dev, out, stream=ms)
            sink = torch.zeros(256, dtype=torch.float32, device="cuda")
            probe.synthetic_compute(ms, 64, 1000, sink)
            ms.close()  # waits for the stream
            assert_same_bits(out, want, f"masked stream, {len(cus)} CUs")
            assert float(sink.sum()) > 0
        with pytest.raises(z.ZcgError) as e:  # a mask with no compute unit of the device
            z.stream_create_cu_mask([])
        assert e.value.status == -1
        with pytest.raises(z.ZcgError) as e:  # a die left without compute units: the runtime refuses
            z.stream_create_cu_mask([0])
        assert e.value.status == -4
        z.gather(table, idx_dev, out)  # the refusal leaves no error behind
        torch.cuda.synchronize()
    finally:
        table.close()


ORDERED_SHAPES = [(40000, 16, "f16"), (40000, 16, "f32"), (30000, 64, "f16"), (5000, 100, "f32"),
                  (3000, 602, "f32"), (2000, 257, "f16"), (900, 1025, "f32"), (1001, 3, "f32")]


@pytest.mark.parametrize("n_rows,dim,dtype", ORDERED_SHAPES)
def test_ordered_gather_matches_oracle(n_rows, dim, dtype):
    """Processing order changes which work item moves which row, never the result."""
    table = host_table(n_rows, dim, dtype, seed=dim)
    try:
        idx = wl.uniform_indices(50021, n_rows, seed=17)  # many repeated and adjacent rows
        want = oracle_gather(table.host_array(), idx)
        idx_dev = torch.from_numpy(idx).cuda()
        ws_bytes = z.order_workspace_bytes(idx.size)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        order = torch.empty(idx.size, dtype=torch.int64, device="cuda")
        z.make_order(idx_dev, n_rows, order, ws, ws_bytes)
        torch.cuda.synchronize()
        o = order.cpu().numpy()
        assert np.array_equal(np.sort(o), np.arange(idx.size))  # a permutation
        assert np.array_equal(o, np.argsort(idx, kind="stable"))  # ascending, ties in list order
        for name, perm in (("sorted", order),
                           ("random", torch.randperm(idx.size, device="cuda")),
                           ("reversed", torch.arange(idx.size - 1, -1, -1, device="cuda"))):
            for variant in (z.VARIANT_AUTO, z.VARIANT_ROWVEC, z.VARIANT_ALIGNED, z.VARIANT_HALFLINE):
                out = torch.full((idx.size, dim), -7.0, dtype=TORCH_DT[dtype], device="cuda")
                z.gather_ordered(table, idx_dev, perm, out, z.LaunchOpts(variant=variant))
                torch.cuda.synchronize()
                assert_same_bits(out, want, f"ordered {name} variant={variant}")
        out = torch.zeros((idx.size, dim), dtype=TORCH_DT[dtype], device="cuda")
        with pytest.raises(z.ZcgError) as e:
            z.gather_ordered(table, idx_dev, order, out, z.LaunchOpts(variant=z.VARIANT_NAIVE))
        assert e.value.status == -1
        with pytest.raises(z.ZcgError) as e:
            z.make_order(idx_dev, n_rows, order, ws, ws_bytes - 256)
        assert e.value.status == -1
        z.gather_ordered(table, idx_dev, order, out, n_idx=0)  # empty: nothing to do
    finally:
        table.close()


@pytest.mark.parametrize("n_rows", [1, 2, 31, 256, 257, 65_536, 100_000, 2_450_000, 20_000_000,
                                    (1 << 32) + 5, 1 << 45])
def test_make_order_key_widths_lengths_and_skew(n_rows):
    """The order builder against numpy's stable argsort: 1 to 46 key bits (one to six digit
    passes; beyond 32 bits the keys are looked up again in the list), list lengths from one entry
    to several tiles per block and beyond 4 M entries (longer stretches per wavefront), uniform,
    constant, two-valued and ascending / descending lists."""
    rng = np.random.default_rng(n_rows % 1000003)
    lengths = [1, 2, 63, 64, 65, 1023, 4096, 4097, 50_021, 300_000]
    if n_rows in (257, 20_000_000):
        lengths.append(4_500_000)
    for n in lengths:
        lists = {"uniform": rng.integers(0, n_rows, n)}
        if n in (65, 50_021):
            lists["constant"] = np.full(n, n_rows - 1, np.int64)
            lists["two values"] = np.where(rng.random(n) < 0.9, 0, n_rows - 1).astype(np.int64)
            lists["ascending"] = np.sort(lists["uniform"])
            lists["descending"] = np.sort(lists["uniform"])[::-1].copy()
        ws_bytes = z.order_workspace_bytes(n)
        assert ws_bytes >= 8 * n and ws_bytes % 256 == 0
        ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
        ws_ptr = (ws.data_ptr() + 255) // 256 * 256
        for name, idx in lists.items():
            idx_dev = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int64)).cuda()
            order = torch.full((n + 2,), -5, dtype=torch.int64, device="cuda")  # guard entries
            z.make_order(idx_dev, n_rows, order[1:], ws_ptr, ws_bytes, n_idx=n)
            torch.cuda.synchronize()
            o = order.cpu().numpy()
            assert o[0] == -5 and o[-1] == -5, f"{name} n={n}: wrote outside the order array"
            assert np.array_equal(o[1:-1], np.argsort(idx, kind="stable")), f"{name} n={n} n_rows={n_rows}"


def test_make_order_argument_checks_and_capture():
    n, n_rows = 20_000, 1000
    idx = torch.from_numpy(wl.uniform_indices(n, n_rows, seed=1)).cuda()
    order = torch.empty(n, dtype=torch.int64, device="cuda")
    ws_bytes = z.order_workspace_bytes(n)
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    ws_ptr = (ws.data_ptr() + 255) // 256 * 256
    for bad in (lambda: z.make_order(idx, 0, order, ws_ptr, ws_bytes),
                lambda: z.make_order(idx, n_rows, order, ws_ptr, ws_bytes - 256),
                lambda: z.make_order(idx, n_rows, order, ws_ptr, ws_bytes, n_idx=1 << 32),
                lambda: z.make_order(idx, n_rows, 0, ws_ptr, ws_bytes)):
        with pytest.raises(z.ZcgError) as e:
            bad()
        assert e.value.status == -1
    with pytest.raises(z.ZcgError) as e:
        z.make_order(idx, n_rows, order, ws_ptr + 8, ws_bytes)
    assert e.value.status == -6
    z.make_order(idx, n_rows, order, ws_ptr, ws_bytes, n_idx=0)  # nothing to do
    assert z.order_workspace_bytes(0) == 0
    # a workspace sized for a longer list serves every shorter one, also across the change of
    # tiling at 2^20 entries
    big = (1 << 20) + 1
    big_ws = torch.empty(z.order_workspace_bytes(big), dtype=torch.uint8, device="cuda")
    for m in (big, 1 << 20, (1 << 20) - 1, 70_000):
        lst = torch.from_numpy(wl.uniform_indices(m, 5_000_000, seed=m)).cuda()
        o = torch.empty(m, dtype=torch.int64, device="cuda")
        z.make_order(lst, 5_000_000, o, big_ws, big_ws.numel())
        torch.cuda.synchronize()
        assert np.array_equal(o.cpu().numpy(), np.argsort(lst.cpu().numpy(), kind="stable")), m
    # the build is kernel launches only: it can be captured, and a replay follows the list
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        z.make_order(idx, n_rows, order, ws_ptr, ws_bytes, stream=s)
    for seed in (2, 3, 4):
        fresh = wl.uniform_indices(n, n_rows, seed=seed)
        idx.copy_(torch.from_numpy(fresh))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(order.cpu().numpy(), np.argsort(fresh, kind="stable")), f"replay {seed}"


@pytest.mark.parametrize("n_rows,dim,dtype", [(600_000, 16, "f16"), (400_000, 16, "f32"),
                                               (300_000, 32, "f32"), (250_000, 24, "f32")])
def test_auto_with_lent_workspace_orders_short_rows(n_rows, dim, dtype):
    """zcg_gather_ex, variant AUTO, workspace lent through the options: long lists of
    host-resident rows of at most a line are walked in ascending table order. Same bytes."""
    table = host_table(n_rows, dim, dtype, seed=dim)
    try:
        n = 200_003
        idx = wl.uniform_indices(n, n_rows, seed=23)
        want = oracle_gather(table.host_array(), idx)
        idx_dev = torch.from_numpy(idx).cuda()
        ws_bytes = z.gather_workspace_bytes(n)
        ws = torch.zeros(ws_bytes + 256, dtype=torch.uint8, device="cuda")
        ws_ptr = (ws.data_ptr() + 255) // 256 * 256
        lent = z.LaunchOpts(workspace_dev=ws_ptr, workspace_bytes=ws_bytes)
        out = torch.full((n, dim), -7, dtype=TORCH_DT[dtype], device="cuda")
        assert z.plan_gather(table, n, out, lent)["ordered"] == 1
        assert z.plan_gather(table, n, out)["ordered"] == 0
        assert z.plan_gather(table, 5000, out, lent)["ordered"] == 0
        for rep in range(2):
            out = torch.full((n, dim), -7, dtype=TORCH_DT[dtype], device="cuda")
            z.gather_ex(table, idx_dev, out, lent)
            torch.cuda.synchronize()
            assert_same_bits(out, want, f"auto ordered rep {rep}")
        # order build + gather are kernel launches only: one captured graph, replayed on new lists
        s = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            z.gather_ex(table, idx_dev, out, lent, stream=s)
        for seed in (31, 32):
            fresh = wl.uniform_indices(n, n_rows, seed=seed)
            idx_dev.copy_(torch.from_numpy(fresh))
            out.fill_(-7)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert_same_bits(out, oracle_gather(table.host_array(), fresh), f"replay {seed}")
        idx_dev.copy_(torch.from_numpy(idx))
        out = torch.full((n, dim), -7, dtype=TORCH_DT[dtype], device="cuda")
        z.gather_ex(table, idx_dev, out, lent)
        torch.cuda.synchronize()
        # the order it built is left at the start of the workspace
        off = ws_ptr - ws.data_ptr()
        built = ws[off: off + 8 * n].view(torch.int64).cpu().numpy()
        assert np.array_equal(built, np.argsort(idx, kind="stable"))
        # too little workspace, a forced kernel, a short list: the plain path, same result
        # (a long list that is sparse in its table is left in list order too: next test)
        for opts, n_use in ((z.LaunchOpts(workspace_dev=ws_ptr, workspace_bytes=ws_bytes // 2), n),
                            (z.LaunchOpts(variant=z.VARIANT_ROWVEC, workspace_dev=ws_ptr,
                                          workspace_bytes=ws_bytes), n),
                            (z.LaunchOpts(workspace_dev=ws_ptr, workspace_bytes=ws_bytes), 5000)):
            ws.zero_()
            out = torch.full((n_use, dim), -7, dtype=TORCH_DT[dtype], device="cuda")
            z.gather_ex(table, idx_dev, out, opts, n_idx=n_use)
            torch.cuda.synchronize()
            assert_same_bits(out, want[:n_use], "plain path")
            assert not bool(ws.any())  # the workspace was left alone
        with pytest.raises(z.ZcgError) as e:
            z.gather_ex(table, idx_dev, out, z.LaunchOpts(workspace_bytes=64))
        assert e.value.status == -1
        # a bad option is refused before the order builder touches the workspace
        ws.zero_()
        with pytest.raises(z.ZcgError) as e:
            z.gather_ex(table, idx_dev, out, z.LaunchOpts(workspace_dev=ws_ptr, workspace_bytes=ws_bytes, unroll=3))
        assert e.value.status == -1
        torch.cuda.synchronize()
        assert not bool(ws.any())
        # a workspace that overlaps the list or the table is refused before anything is launched
        for bad_ws in (idx_dev.data_ptr() // 256 * 256, table.device_ptr):
            with pytest.raises(z.ZcgError) as e:
                z.gather_ex(table, idx_dev, out, z.LaunchOpts(workspace_dev=bad_ws, workspace_bytes=ws_bytes))
            assert e.value.status == -7
    finally:
        table.close()


def test_auto_leaves_sparse_lists_in_list_order():
    """200 k entries over 12 M rows of 32 bytes: an eighth of a listed row per 256-byte pair, too
    few shared requests to pay for building the order; the workspace stays untouched."""
    n_rows, dim, n = 12_000_000, 16, 200_003
    table = host_table(n_rows, dim, "f16", seed=3)
    try:
        idx = wl.uniform_indices(n, n_rows, seed=29)
        idx_dev = torch.from_numpy(idx).cuda()
        ws_bytes = z.gather_workspace_bytes(n)
        ws = torch.zeros(ws_bytes, dtype=torch.uint8, device="cuda")
        out = torch.full((n, dim), -7, dtype=torch.float16, device="cuda")
        lent = z.LaunchOpts(workspace_dev=ws.data_ptr(), workspace_bytes=ws_bytes)
        assert z.plan_gather(table, n, out, lent)["ordered"] == 0
        z.gather_ex(table, idx_dev, out, lent)
        torch.cuda.synchronize()
        assert_same_bits(out, oracle_gather(table.host_array(), idx), "sparse list")
        assert not bool(ws.any())
    finally:
        table.close()


def test_seeded_random_shapes_knobs_and_offsets():
    """40 seeded random combinations of row size, dtype, list length, base offsets, kernel and
    launch knobs (ordered or not) against the oracle; one long list to exercise grid striding."""
    rng = np.random.default_rng(20210303)
    cases = []
    for _ in range(40):
        dtype = str(rng.choice(["f16", "f32", "f32", "i8", "f64"]))
        elem = {"i8": 1, "f16": 2, "f32": 4, "f64": 8}[dtype]
        dim = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 64, 100, 127, 128, 129, 255, 300, 602, 1000, 2051]))
        n_rows = int(rng.integers(1, 4000))
        n_idx = int(rng.choice([1, 2, 63, 64, 65, 1000, 4097, 30000]))
        cases.append((dtype, elem, dim, n_rows, n_idx))
    cases.append(("f32", 4, 2, 100_000, 3_000_000))  # 8-byte rows, long list
    for ci, (dtype, elem, dim, n_rows, n_idx) in enumerate(cases):
        t_off = int(rng.integers(0, 9)) * elem  # table base off by 0..8 elements
        o_off = int(rng.integers(0, 9)) * elem
        backing = z.alloc_table(n_rows + 1, dim + 16, dtype)  # room for the shifted view
        try:
            wl.fill_table_ptr(backing.host_ptr, n_rows + 1, dim + 16, dtype, seed=ci, mode=wl.FILL_RAW_BITS)
            flat = backing.host_array().reshape(-1)
            sub = np.ascontiguousarray(flat[t_off // elem: t_off // elem + n_rows * dim].reshape(n_rows, dim))
            view = z.table_from_device(backing.device_ptr + t_off, n_rows, dim, dtype)
            idx = rng.integers(0, n_rows, n_idx)
            want = oracle_gather(sub, idx)
            idx_dev = torch.from_numpy(idx).cuda()
            buf = torch.zeros(n_idx * dim + 32, dtype=TORCH_DT[dtype], device="cuda")
            out = buf[o_off // elem: o_off // elem + n_idx * dim].view(n_idx, dim)
            opts = z.LaunchOpts(variant=int(rng.integers(0, 5)), unroll=int(rng.choice([0, 1, 2, 4, 8])),
                                line_bytes=int(rng.choice([0, 32, 64, 128, 256])),
                                vec_bytes=int(rng.choice([0] + [v for v in (1, 2, 4, 8, 16) if v >= elem])),
                                group_lanes=int(rng.choice([0, 1, 8, 64])),
                                shifted_stores=int(rng.integers(0, 3)), nt_loads=int(rng.integers(0, 4)),
                                nt_stores=int(rng.integers(0, 3)),
                                max_blocks=int(rng.choice([0, 1, 7, 300])),
                                row_splits=int(rng.choice([0, 1, 2, 5])),
                                half_ends=int(rng.integers(0, 3)))
            what = f"case {ci}: {dtype} dim={dim} rows={n_rows} n_idx={n_idx} t_off={t_off} o_off={o_off} " \
                   f"opts={[getattr(opts, f) for f, _ in opts._fields_]}"
            if rng.random() < 0.4 and opts.variant != z.VARIANT_NAIVE:
                perm = torch.randperm(n_idx, device="cuda")
                z.gather_ordered(view, idx_dev, perm, out, opts)
                what += " ordered"
            else:
                z.gather_ex(view, idx_dev, out, opts)
            torch.cuda.synchronize()
            assert_same_bits(out, want, what)
            guard_lo, guard_hi = buf[: o_off // elem], buf[o_off // elem + n_idx * dim:]
            as_int = {1: torch.int8, 2: torch.int16, 4: torch.int32, 8: torch.int64}[elem]
            assert not bool(guard_lo.view(as_int).any()), what
            assert not bool(guard_hi.view(as_int).any()), what
            view.close()
        finally:
            backing.close()


def test_seeded_random_cases_on_host_resident_views_hbm_copies_and_lent_workspace():
    """400 seeded random cases: element size, row length (up to 280 KB), list length, table and
    output offsets, where the table lives (a host-resident view, the same memory flagged as a
    device table, a copy in HBM), default or random launch options, a caller's order or lent
    workspace; every output byte against the oracle, guard elements around the output."""
    rng = np.random.default_rng(20210304)
    as_int = {1: torch.int8, 2: torch.int16, 4: torch.int32, 8: torch.int64}
    for ci in range(400):
        dtype = str(rng.choice(["f16", "f32", "f32", "i8", "f64"]))
        elem = {"i8": 1, "f16": 2, "f32": 4, "f64": 8}[dtype]
        r = rng.random()
        dim = int(rng.integers(1, 200)) if r < 0.5 else (int(rng.integers(1, 1400)) if r < 0.9 else
                                                         int(rng.choice([4096, 5000, 16384, 20001, 70000])))
        n_rows = int(rng.integers(1, 3000)) if dim < 3000 else int(rng.integers(1, 60))
        n_idx = (int(rng.choice([1, 2, 3, 63, 64, 65, 127, 129, 1000, 4097, 30000, 70000])) if dim < 3000
                 else int(rng.choice([1, 2, 5, 33, 100])))
        t_off = int(rng.integers(0, 70)) * elem if rng.random() < 0.7 else 0
        o_off = int(rng.integers(0, 40)) * elem if rng.random() < 0.7 else 0
        mode = str(rng.choice(["view", "device table over host memory", "hbm"]))
        pad_rows = (t_off + dim * elem - 1) // (dim * elem) + 1
        backing = z.alloc_table(n_rows + pad_rows, dim, dtype)
        view = None
        try:
            wl.fill_table_ptr(backing.host_ptr, n_rows + pad_rows, dim, dtype, seed=ci, mode=wl.FILL_RAW_BITS)
            flat = backing.host_array().reshape(-1)
            sub = np.ascontiguousarray(flat[t_off // elem: t_off // elem + n_rows * dim].reshape(n_rows, dim))
            if mode == "view":
                view = z.table_view(backing, t_off, n_rows, dim, dtype)
            elif mode == "hbm":
                keep = torch.zeros(n_rows * dim + 80, dtype=TORCH_DT[dtype], device="cuda")
                keep[t_off // elem: t_off // elem + n_rows * dim] = torch.from_numpy(sub.reshape(-1)).cuda()
                view = z.table_from_device(keep.data_ptr() + t_off, n_rows, dim, dtype)
            else:
                view = z.table_from_device(backing.device_ptr + t_off, n_rows, dim, dtype)
            idx = rng.integers(0, n_rows, n_idx)
            if rng.random() < 0.2:
                idx = np.sort(idx)
            want = oracle_gather(sub, idx)
            idx_dev = torch.from_numpy(idx).cuda()
            buf = torch.zeros(n_idx * dim + 64, dtype=TORCH_DT[dtype], device="cuda")
            out = buf[o_off // elem: o_off // elem + n_idx * dim].view(n_idx, dim)
            opts = z.LaunchOpts()
            if rng.random() < 0.55:
                opts = z.LaunchOpts(variant=int(rng.integers(0, 5)), unroll=int(rng.choice([0, 1, 2, 4, 8])),
                                    line_bytes=int(rng.choice([0, 32, 64, 128, 256])),
                                    vec_bytes=int(rng.choice([0] + [v for v in (1, 2, 4, 8, 16) if v >= elem])),
                                    group_lanes=int(rng.choice([0, 1, 2, 4, 8, 16, 32, 64])),
                                    shifted_stores=int(rng.integers(0, 3)), nt_loads=int(rng.integers(0, 4)),
                                    nt_stores=int(rng.integers(0, 3)),
                                    max_blocks=int(rng.choice([0, 1, 7, 300, 5000])),
                                    row_splits=int(rng.choice([0, 1, 2, 5, 64])), half_ends=int(rng.integers(0, 3)))
            what = (f"case {ci}: {dtype} dim={dim} rows={n_rows} n_idx={n_idx} t_off={t_off} o_off={o_off} "
                    f"{mode} opts={[getattr(opts, f) for f, _ in opts._fields_][:11]}")
            r = rng.random()
            if r < 0.3 and opts.variant != z.VARIANT_NAIVE:
                z.gather_ordered(view, idx_dev, torch.randperm(n_idx, device="cuda"), out, opts)
                what += " with an order"
            elif r < 0.5 and opts.variant == z.VARIANT_AUTO:
                ws_bytes = z.gather_workspace_bytes(n_idx)
                ws = torch.zeros(ws_bytes + 256, dtype=torch.uint8, device="cuda")
                opts.workspace_dev = ws.data_ptr() + (-ws.data_ptr()) % 256
                opts.workspace_bytes = ws_bytes
                z.gather_ex(view, idx_dev, out, opts)
                what += " with lent workspace"
            else:
                z.gather_ex(view, idx_dev, out, opts)
            torch.cuda.synchronize()
            assert_same_bits(out, want, what)
            assert not bool(buf[: o_off // elem].view(as_int[elem]).any()), what
            assert not bool(buf[o_off // elem + n_idx * dim:].view(as_int[elem]).any()), what
        finally:
            if view is not None:
                view.close()
            backing.close()


def test_link_probes_give_sane_numbers():
    rtt = probe.measure_host_read_latency(4000)
    assert 0.2 < rtt < 50.0  # microseconds per dependent read of mapped host memory
    assert 5.0 < probe.measure_h2d(64 << 20, 3) < 200.0  # GB/s
    assert 5.0 < probe.measure_host_stream_read(64 << 20, 3) < 200.0  # GB/s
    with pytest.raises(probe.ProbeError):
        probe.measure_host_stream_read(1000, 3)  # not a multiple of a page
    a = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    b = torch.zeros_like(a)
    probe.device_copy(b, a, a.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("flags", [z.ALLOC_DEFAULT, z.ALLOC_NONCOHERENT])
def test_host_updates_between_gathers_are_seen(flags):
    """The table lives in host memory: rows the CPU rewrites after one gather has finished must be
    what the next gather returns, for every kernel (vector caches and the scalar cache alike)."""
    n_rows, dim = 3000, 602
    table = host_table(n_rows, dim, "f32", seed=3, flags=flags)
    try:
        host = table.host_array()
        idx = wl.uniform_indices(9000, n_rows, seed=8)
        idx_dev = torch.from_numpy(idx).cuda()
        for variant in ALL_VARIANTS:
            for round_ in range(3):
                out = torch.zeros((idx.size, dim), dtype=torch.float32, device="cuda")
                z.gather_variant(table, idx_dev, out, variant)
                torch.cuda.synchronize()
                assert_same_bits(out, oracle_gather(host, idx), f"variant {variant} round {round_}")
                host[:] = host[::-1].copy() if round_ % 2 == 0 else host * np.float32(0.5)
    finally:
        table.close()


@pytest.mark.parametrize("n_rows,dim,dtype", [(40, 70_001, "f32"), (24, 65_536, "f16"), (16, 300_003, "i8"),
                                               (12, 40_000, "f64")])
def test_very_wide_rows_and_first_last_row(n_rows, dim, dtype):
    """Rows of hundreds of KB (many passes per wave) and lists that name only the first and
    the last row of the table, for every kernel; also ordered."""
    table = host_table(n_rows, dim, dtype, seed=dim)
    try:
        host = table.host_array()
        lists = [np.array([n_rows - 1], np.int64), np.array([0], np.int64),
                 np.array([n_rows - 1, 0, n_rows - 1, 0, 1], np.int64),
                 wl.uniform_indices(67, n_rows, seed=3)]
        probe = torch.zeros((1, dim), dtype=TORCH_DT[dtype], device="cuda")
        assert z.plan_gather(table, 1, probe)["row_splits"] > 1  # a short list of long rows is split
        assert z.plan_gather(table, 1_000_000, probe)["row_splits"] == 1
        for idx in lists:
            want = oracle_gather(host, idx)
            for variant in ALL_VARIANTS:
                for splits in (0, 1, 13):
                    got = run_gather(table, idx, dtype, z.LaunchOpts(variant=variant, row_splits=splits))
                    assert_same_bits(got, want, f"{dtype} dim={dim} n_idx={len(idx)} variant={variant} splits={splits}")
            idx_dev = torch.from_numpy(idx).cuda()
            order = torch.from_numpy(np.argsort(idx, kind="stable")).cuda()
            out = torch.zeros((len(idx), dim), dtype=TORCH_DT[dtype], device="cuda")
            z.gather_ordered(table, idx_dev, order, out)
            torch.cuda.synchronize()
            assert_same_bits(out, want, f"ordered {dtype} dim={dim} n_idx={len(idx)}")
    finally:
        table.close()


@pytest.mark.parametrize("resident", ["host", "hbm"])
def test_lists_of_more_than_2_31_entries(resident):
    """Positions in the list beyond 2^31 and 2^32 output bytes: 2^31 + 70,001 two-byte rows (a
    17 GB list held in HBM). Checked against the oracle on three stretches of a million entries
    (first, last, around 2^31) and, as a property over every entry, against the library's own
    indexing of the same table in chunks."""
    n_rows, dim, n_idx = 60_000, 1, (1 << 31) + 70_001
    host = host_table(n_rows, dim, "f16", seed=91, mode=wl.FILL_RAW_BITS)
    table_np = host.host_array().copy()
    dev_copy = torch.from_numpy(table_np).cuda()
    table = host if resident == "host" else z.table_from_device(dev_copy.data_ptr(), n_rows, dim, "f16")
    try:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(20310331)
        idx = torch.randint(0, n_rows, (n_idx,), dtype=torch.int64, device="cuda", generator=gen)
        idx[0], idx[-1], idx[1 << 31] = n_rows - 1, 0, n_rows - 1
        out = torch.full((n_idx, dim), -7, dtype=torch.float16, device="cuda")
        z.gather(table, idx, out)
        torch.cuda.synchronize()
        for lo in (0, (1 << 31) - 500_000, n_idx - 1_000_000):
            part = idx[lo:lo + 1_000_000].cpu().numpy()
            assert_same_bits(out[lo:lo + 1_000_000], oracle_gather(table_np, part), f"entries from {lo}")
        bits, table_bits = out.view(torch.int16).view(-1), dev_copy.view(torch.int16).view(-1)
        step = 1 << 28
        for lo in range(0, n_idx, step):
            assert torch.equal(bits[lo:lo + step], table_bits[idx[lo:lo + step]]), f"chunk at {lo}"
    finally:
        if table is not host:
            table.close()
        host.close()
