"""GPU: the gather as a building block of a serving / training loop.

* captured in a HIP graph and replayed: zcg_gather allocates nothing, synchronises nothing and
  never reads the index list on the host, so a replay must pick up whatever the index buffer and
  the host table hold at replay time (Section 3.3: the list is produced anew for every minibatch);
* issued from several host threads on several streams at once against one table handle;
* with the index list itself left in mapped pinned host memory (no host-to-device copy at all).

Every result is compared bit for bit with the CPU oracle.
"""
import threading

import numpy as np
import pytest

import zcg_workload as wl
from oracle import gather as oracle_gather

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
z = pytest.importorskip("paper_2103_03330_amd")


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)


def _table(n_rows, dim, dtype="f32", seed=7):
    t = z.alloc_table(n_rows, dim, dtype)
    wl.fill_table_ptr(t.host_ptr, n_rows, dim, dtype, seed=seed)
    return t


@pytest.mark.parametrize("dim,variant", [(100, z.VARIANT_AUTO), (100, z.VARIANT_NAIVE),
                                         (602, z.VARIANT_AUTO), (16, z.VARIANT_AUTO)])
def test_graph_replay_follows_index_buffer_and_table(dim, variant):
    _need_gpu()
    n_rows, n_idx = 40_000, 9_001
    table = _table(n_rows, dim)
    host = table.host_array()
    idx_dev = torch.zeros(n_idx, dtype=torch.int64, device="cuda")
    out = torch.zeros((n_idx, dim), dtype=torch.float32, device="cuda")
    lists = [wl.uniform_indices(n_idx, n_rows, seed=100 + r) for r in range(4)]
    try:
        # eager result first (also warms everything the capture must not initialise)
        idx_dev.copy_(torch.from_numpy(lists[0]))
        z.gather_variant(table, idx_dev, out, variant)
        torch.cuda.synchronize()
        assert out.cpu().numpy().tobytes() == oracle_gather(host, lists[0]).tobytes()

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            z.gather_variant(table, idx_dev, out, variant, stream=torch.cuda.current_stream())
        for r in range(1, 4):
            # eager work and synchronisation between the replays, as a real loop has
            idx_dev.copy_(torch.from_numpy(lists[r]))
            host[lists[r][0]] += 1.0  # the host rewrites a row the next replay must see
            out.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            want = oracle_gather(host, lists[r])
            assert out.cpu().numpy().tobytes() == want.tobytes(), f"replay {r}"
        del graph
    finally:
        torch.cuda.synchronize()
        table.close()


def test_graph_with_ordered_gather():
    """The ordered gather captured; the order is rebuilt eagerly for every new list (the
    library sort is kept out of the graph), the workspace is the caller's."""
    _need_gpu()
    n_rows, dim, n_idx = 30_000, 16, 20_000
    table = _table(n_rows, dim, "f16", seed=3)
    host = table.host_array()
    idx_dev = torch.zeros(n_idx, dtype=torch.int64, device="cuda")
    order = torch.zeros(n_idx, dtype=torch.int64, device="cuda")
    ws_bytes = z.order_workspace_bytes(n_idx)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device="cuda")
    assert ws.data_ptr() % 256 == 0
    out = torch.zeros((n_idx, dim), dtype=torch.float16, device="cuda")
    lists = [wl.uniform_indices(n_idx, n_rows, seed=200 + r) for r in range(3)]
    try:
        idx_dev.copy_(torch.from_numpy(lists[0]))
        z.make_order(idx_dev, n_rows, order, ws, ws_bytes)
        z.gather_ordered(table, idx_dev, order, out)
        torch.cuda.synchronize()
        assert out.cpu().numpy().tobytes() == oracle_gather(host, lists[0]).tobytes()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            z.gather_ordered(table, idx_dev, order, out, stream=torch.cuda.current_stream())
        for r in range(1, 3):
            idx_dev.copy_(torch.from_numpy(lists[r]))
            z.make_order(idx_dev, n_rows, order, ws, ws_bytes)
            out.zero_()
            torch.cuda.synchronize()
            perm = order.cpu().numpy()
            assert np.array_equal(np.sort(perm), np.arange(n_idx))
            assert np.all(np.diff(lists[r][perm]) >= 0)
            graph.replay()
            torch.cuda.synchronize()
            assert out.cpu().numpy().tobytes() == oracle_gather(host, lists[r]).tobytes(), f"replay {r}"
        del graph
    finally:
        torch.cuda.synchronize()
        table.close()


def test_threads_and_streams_share_one_table():
    _need_gpu()
    n_rows, dim, n_threads, rounds = 60_000, 100, 4, 12
    table = _table(n_rows, dim, seed=11)
    host = table.host_array()
    errors, lock = [], threading.Lock()

    def worker(tid):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            for r in range(rounds):
                n_idx = 1 + (tid * 7919 + r * 104729) % 30_000
                idx = wl.uniform_indices(n_idx, n_rows, seed=1000 * tid + r)
                with torch.cuda.stream(stream):
                    idx_dev = torch.from_numpy(idx).to("cuda", non_blocking=False)
                    out = torch.empty((n_idx, dim), dtype=torch.float32, device="cuda")
                    z.gather(table, idx_dev, out, stream=stream)
                stream.synchronize()
                if out.cpu().numpy().tobytes() != oracle_gather(host, idx).tobytes():
                    raise AssertionError(f"thread {tid} round {r} n_idx {n_idx}: mismatch")
        except Exception as exc:  # noqa: BLE001 - reported by the main thread
            with lock:
                errors.append(repr(exc))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(n_threads)]
    try:
        for t in threads:
            t.start()
        for t in threads:
            t.join(timeout=120)
        assert not any(t.is_alive() for t in threads), "a worker did not finish"
        assert not errors, errors
    finally:
        torch.cuda.synchronize()
        table.close()


def test_index_list_in_mapped_host_memory():
    """The list may stay in pinned, GPU-mapped host memory: the kernel then reads it over the
    link as well (8 bytes per row). An int64 one-column table is such an allocation."""
    _need_gpu()
    n_rows, dim, n_idx = 50_000, 100, 12_345
    table = _table(n_rows, dim, seed=13)
    idx_buf = z.alloc_table(n_idx, 1, "f64")  # any 8-byte element type
    try:
        idx = wl.uniform_indices(n_idx, n_rows, seed=77)
        idx_buf.host_array().view(np.int64).reshape(-1)[:] = idx
        out = torch.zeros((n_idx, dim), dtype=torch.float32, device="cuda")
        z.gather(table, idx_buf.device_ptr, out, n_idx=n_idx)
        torch.cuda.synchronize()
        assert out.cpu().numpy().tobytes() == oracle_gather(table.host_array(), idx).tobytes()
        assert z.validate_indices(table, idx_buf.device_ptr, n_idx=n_idx) == 0
    finally:
        torch.cuda.synchronize()
        idx_buf.close()
        table.close()
