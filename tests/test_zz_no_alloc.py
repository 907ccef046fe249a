"""GPU: zcg_make_order_static, the entry point that allocates nothing (its temporary memory is a
static device array of the library), against zcg_make_order with a caller workspace: the same
order bit for bit, on calls in a row that share the array, the later ones smaller."""
import numpy as np
import pytest

import zcg_workload as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
z = pytest.importorskip("paper_2103_03330_amd")


def reference_order(idx_dev, n, n_rows):
    ws_bytes = z.order_workspace_bytes(n)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    order = torch.empty(n, dtype=torch.int64, device="cuda")
    z.make_order(idx_dev, n_rows, order, ws, ws_bytes, n_idx=n)
    torch.cuda.synchronize()
    return order.cpu().numpy()


def test_static_scratch_order_matches_workspace_order():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    z.load_library()
    lib = z.load_library()
    # (n_idx, n_rows): the largest size first, then smaller calls that find the array used
    cases = [(z.STATIC_ORDER_MAX_IDX, 10_000_000), (300_007, 2_450_000), (4097, 100_000), (1, 5),
             (70_001, (1 << 33) + 11), (z.STATIC_ORDER_MAX_IDX, 1 << 40)]
    for n, n_rows in cases:
        print(f"zcg_make_order_static n_idx={n} n_rows={n_rows}", flush=True)
        idx = np.random.default_rng(n).integers(0, n_rows, n)
        idx_dev = torch.from_numpy(idx).cuda()
        order = torch.full((n + 2,), -9, dtype=torch.int64, device="cuda")
        rc = lib.zcg_make_order_static(idx_dev.data_ptr(), n, n_rows, order[1:].data_ptr(), None)
        assert rc == 0, z.strerror(rc)
        torch.cuda.synchronize()
        got = order.cpu().numpy()
        assert got[0] == -9 and got[-1] == -9
        want = reference_order(idx_dev, n, n_rows)
        assert np.array_equal(got[1:-1], want), f"n_idx={n} n_rows={n_rows}"
        assert np.array_equal(want, np.argsort(idx, kind="stable"))
    # sizes beyond the array, and the usual argument errors, are refused before any launch
    idx_dev = torch.zeros(8, dtype=torch.int64, device="cuda")
    order = torch.zeros(8, dtype=torch.int64, device="cuda")
    assert lib.zcg_make_order_static(idx_dev.data_ptr(), z.STATIC_ORDER_MAX_IDX + 1, 100, order.data_ptr(), None) == -12
    assert "capacity" in z.strerror(-12)
    assert lib.zcg_make_order_static(idx_dev.data_ptr(), -1, 100, order.data_ptr(), None) == -1
    assert lib.zcg_make_order_static(idx_dev.data_ptr(), 8, 0, order.data_ptr(), None) == -1
    assert lib.zcg_make_order_static(None, 8, 100, order.data_ptr(), None) == -1
    assert lib.zcg_make_order_static(idx_dev.data_ptr() + 4, 4, 100, order.data_ptr(), None) == -6
    assert lib.zcg_make_order_static(None, 0, 100, None, None) == 0
    # no allocation, only kernel launches: the call can be captured in a graph, where an
    # allocation would be refused; replays follow the list's current contents
    n, n_rows = 50_021, 777_777
    idx_dev = torch.from_numpy(wl.uniform_indices(n, n_rows, seed=1)).cuda()
    order = torch.empty(n, dtype=torch.int64, device="cuda")
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        z.make_order_static(idx_dev, n_rows, order, stream=s)
    for seed in (2, 3):
        fresh = wl.uniform_indices(n, n_rows, seed=seed)
        idx_dev.copy_(torch.from_numpy(fresh))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(order.cpu().numpy(), np.argsort(fresh, kind="stable")), f"replay {seed}"
    # and it feeds the ordered gather like any other order
    table = z.alloc_table(n_rows, 16, "f16")
    try:
        wl.fill_table_ptr(table.host_ptr, n_rows, 16, "f16", seed=9)
        out = torch.zeros((n, 16), dtype=torch.float16, device="cuda")
        z.gather_ordered(table, idx_dev, order, out)
        torch.cuda.synchronize()
        assert out.cpu().numpy().tobytes() == table.host_array()[fresh].tobytes()
    finally:
        table.close()
